// Fused execution path of libLOT: the whole LOT attention forward in one persistent kernel.
//
// Work decomposition.  A "pair" is one (batch*head problem, side) with side 0 = keys and
// side 1 = queries; the two Sinkhorn solves of a problem are independent until the very end
// (paper, Method: the two entropic problems share only Z, beta and eps).  Each pair is split
// over `cluster` workgroups ("chunks" of consecutive 32-token tiles).  A workgroup has four
// wavefronts; a wavefront owns every fourth tile of the chunk.
//
// One Sinkhorn iteration is ONE pass over the chunk's tokens.  For a tile of 32 tokens the
// similarities C^T (pivots x tokens) come out of MFMA with the pivots as the M dimension, the
// current pivot potential g added for free through the accumulator input, so that a lane owns
// one token and 16*RB of its pivots:
//     m_i = max_t (C_it + g_t),  e_it = exp((C_it + g_t - m_i)/eps),  s_i = sum_t e_it
// is the token-side update (f_i is implicit: a_i e_it / s_i is the coupling after it), and the
// pivot-side update needs only the column sums of e_it / s_i, accumulated per lane across the
// tiles and reduced once per pass: lanes -> wavefront -> workgroup (LDS) -> cluster (global
// partials in a fixed order, so results are bit-reproducible):
//     g_t += eps * log(n beta_t / sum_i e_it/s_i).
// The last key-side pass also accumulates U = sum_j (e_jt/s_j) V_j with MFMA (the coupling tile
// is transposed through LDS), giving Y'_t = U_t / colsum_t = (Gamma2 V)_t / beta_t.  The query
// side runs one more pass that rebuilds its coupling tile and multiplies it with
// Y''_t = n beta_t/colsum_t * Y'_t by MFMA to write O (paper: "Rank and complexity", factored
// apply O = Gamma1 (Diag(beta)^-1 (Gamma2 V)), times n so that the attention matrix is doubly
// stochastic).  lot_couplings runs the same passes and stores the coupling tiles instead.
//
// Cross-workgroup waits are bounded: a wait that exceeds its poll budget raises the status word
// in the workspace and the workgroup leaves the kernel, so every wavefront always exits.
#include <cmath>

#include "lot_internal.h"
#include "lot_tile.h"

namespace lot {
namespace {


enum { EPI_NONE = 0, EPI_ACCUM_U = 1, EPI_EXPAND = 2, EPI_GAMMA = 3 };
enum { MODE_ATTENTION = 0, MODE_COUPLINGS = 1 };

// Developer instrumentation (compiled out unless LOT_TRACE is defined): thread 0 of every workgroup
// stamps the constant-rate clock into slot `slot` of its 128-slot record, kept in the last 8 MiB of
// the workspace (a region only the reference path uses).
#ifdef LOT_TRACE
#define LOT_STAMP(slot) do { if (threadIdx.x == 0 && (slot) < 128 && p.trace) p.trace[(size_t)blockIdx.x * 128 + (slot)] = wall_clock64(); } while (0)
#else
#define LOT_STAMP(slot) do { } while (0)
#endif

struct FusedParams {
    const void* Q;
    const void* K;
    const void* V;
    const float* Z;
    const float* beta;
    void* out;
    float* gamma1;
    float* gamma2;
    unsigned long long* status;   // [0] = nonce of a launch in which a wait gave up, [1] = nonce of the last launch
    uint32_t* arrive;     // [G]: workgroups that have posted their share of U
    uint32_t* yready;     // [G]
    unsigned long long* cleared;   // [G]: holds this launch's nonce once the problem's counters are zero
    unsigned long long nonce;
    unsigned long long* colacc;   // [G][2 sides][2 parities][64]: count << 56 | fixed-point column sum
    float* u_part;        // [G][cluster_cap][64][D]
    float* y_tile;        // [G][64][D]
    int G, H, r;
    // per side (0 = keys and values, 1 = queries and the output):
    int n_side[2];          // tokens per problem
    int stride_side[2];     // tokens between consecutive problems in memory (>= n_side)
    int tpw_side[2];        // tiles per workgroup
    const float* mass_side[2];   // [G][n_side] token masses, or null: uniform 1/n_side
    int cluster, cluster_cap, num_items, iters, mode;
    float eps;
    float fx_scale, fx_unscale;   // 2^F and 2^-F of the fixed-point column sums
    uint32_t spin_limit;
    unsigned long long* trace;   // LOT_TRACE builds only
};

// Poll *counter until it reaches target.  Thread 0 only.  False if the budget ran out or another
// workgroup already gave up.
__device__ inline bool gave_up(const unsigned long long* status, unsigned long long nonce)
{
    return __hip_atomic_load(status, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == nonce;
}
__device__ inline void give_up(unsigned long long* status, unsigned long long nonce)
{
    __hip_atomic_store(status, nonce, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ inline bool spin_until(uint32_t* counter, uint32_t target, const unsigned long long* status,
                                  unsigned long long nonce, uint32_t limit)
{
    for (uint32_t k = 0; k < limit; ++k) {
        if (__hip_atomic_load(counter, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) >= target) return true;
        if ((k & 63u) == 63u && gave_up(status, nonce)) return false;
        __builtin_amdgcn_s_sleep(1);
    }
    return false;
}



// ---------------------------------------------------------------------------------------------
// one pass over this wavefront's tiles
// ---------------------------------------------------------------------------------------------
// fp32 I/O: the similarities are six bf16 products over pieces of the operands (pivot pieces in LDS)
// instead of fp32 MFMAs.
template <typename IO, int D, int RB, int WAVES>
constexpr bool similarity_by_pieces() { return io_is_f32<IO>::value; }

template <typename IO, int D, int RB, int EPI, int WAVES>
__device__ __forceinline__ void run_pass(
    const FusedParams& p, const IO* __restrict__ X, const IO* __restrict__ Xnext, int next_side,
    Frag<IO, D>& xfirst, float& mfirst,
    int g, int side, const int (&tile_begins)[2], int tile_end, int lane, int wave, float c1,
    const Frag<IO, D> (&zf)[RB], const void* zlds, const float* glds, f32x16 (&cs)[RB],
    const IO* __restrict__ V, f32x16 (&U)[RB][D / 32], uint16_t* tr_hi, uint16_t* tr_lo,
    const bf16x8* yf_hi, const bf16x8* yf_lo, IO* __restrict__ out)
{
    constexpr int NB = D / 32;
    const int i = lane & 31, kg = lane >> 5;
    const int n = p.n_side[side];
    const int stride = p.stride_side[side];
    const int tile_begin = tile_begins[side];
    // token masses times n (1 for uniform masses): they weight the column sums, the reduction over the
    // keys and the couplings, but not the rows of the attention matrix
    const float* const mass = p.mass_side[side];
    int tile = tile_begin + wave;
    if (tile >= tile_end) {
        // Nothing to do on this side (the two sides can have different numbers of tiles), but the next
        // pass still expects its first tile in xfirst.
        if (Xnext != nullptr) {
            const int nn = p.n_side[next_side];
            const int tok = min((tile_begins[next_side] + wave) * kTileTokens + i, nn - 1);
            load_tokens<D>(xfirst, Xnext + ((size_t)g * p.stride_side[next_side] + tok) * D, kg);
            const float* const mass_next = p.mass_side[next_side];
            mfirst = mass_next ? (float)nn * as_global(mass_next)[(size_t)g * nn + tok] : 1.f;
        }
        return;
    }

    // the first tile's rows were loaded before the previous pass ended (xfirst); the last
    // iteration below loads the first tile of the NEXT pass (same tile range, rows of Xnext),
    // so that no pass starts with an exposed round trip to memory
    Frag<IO, D> xc = xfirst;
    float mcur = mfirst;
    for (; tile < tile_end; tile += WAVES) {
        Frag<IO, D> xn = xc;
        float mnext = mcur;
        if (tile + WAVES < tile_end) {
            const int tok = min((tile + WAVES) * kTileTokens + i, n - 1);
            load_tokens<D>(xn, X + ((size_t)g * stride + tok) * D, kg);
            if (mass) mnext = (float)n * as_global(mass)[(size_t)g * n + tok];
        } else if (Xnext != nullptr) {
            const int nn = p.n_side[next_side];
            const int tok = min((tile_begins[next_side] + wave) * kTileTokens + i, nn - 1);
            load_tokens<D>(xn, Xnext + ((size_t)g * p.stride_side[next_side] + tok) * D, kg);
            const float* const mass_next = p.mass_side[next_side];
            mnext = mass_next ? (float)nn * as_global(mass_next)[(size_t)g * nn + tok] : 1.f;
        }

        // the value rows this tile will be multiplied with are requested now and used at the end
        bf16x8 vh[2][NB], vl[2][NB];
        if (EPI == EPI_ACCUM_U) {
#pragma unroll
            for (int s = 0; s < 2; ++s) {
                const int t0 = tile * kTileTokens + 16 * s + 8 * kg;
                const int left = max(1, min(8, n - t0));
                load_values<D>(vh[s], vl[s], V, (size_t)g * stride + min(t0, n - 1), left, i);
            }
        }

        // The accumulators start from the pivot potentials g_t, read from LDS for every tile (an
        // opaque zero offset keeps the reads inside the loop): holding them in registers for the
        // whole pass costs 16*RB registers that the prefetched tile rows need more.
        int skew = 0;
        asm volatile("" : "+v"(skew));
        f32x16 acc[RB];
        load_pivot_vector<RB>(acc, glds + skew, kg);
        if constexpr (similarity_by_pieces<IO, D, RB, WAVES>()) similarity_pieces<D, RB>(acc, zlds, xc, lane, skew);
        else similarity<D, RB>(acc, zf, xc);

        // token-side update: row maximum, exponentials, row sum
        float m0 = acc[0][0], m1 = acc[0][1], m2 = acc[0][2], m3 = acc[0][3];
#pragma unroll
        for (int mb = 0; mb < RB; ++mb)
#pragma unroll
            for (int j = (mb == 0 ? 4 : 0); j < 16; j += 4) {
                m0 = fmaxf(m0, acc[mb][j]);
                m1 = fmaxf(m1, acc[mb][j + 1]);
                m2 = fmaxf(m2, acc[mb][j + 2]);
                m3 = fmaxf(m3, acc[mb][j + 3]);
            }
        const float m = pair_max(fmaxf(fmaxf(m0, m1), fmaxf(m2, m3)));
        const float mc = m * c1;
        float s0 = 0.f, s1 = 0.f, s2 = 0.f, s3 = 0.f;
#pragma unroll
        for (int mb = 0; mb < RB; ++mb)
#pragma unroll
            for (int j = 0; j < 16; j += 4) {
                const float e0 = exp2_fast(fmaf(acc[mb][j], c1, -mc));
                const float e1 = exp2_fast(fmaf(acc[mb][j + 1], c1, -mc));
                const float e2 = exp2_fast(fmaf(acc[mb][j + 2], c1, -mc));
                const float e3 = exp2_fast(fmaf(acc[mb][j + 3], c1, -mc));
                acc[mb][j] = e0; acc[mb][j + 1] = e1; acc[mb][j + 2] = e2; acc[mb][j + 3] = e3;
                s0 += e0; s1 += e1; s2 += e2; s3 += e3;
            }
        const float s = pair_sum((s0 + s1) + (s2 + s3));
        const int tok = tile * kTileTokens + i;
        const float w = tok < n ? rcp_fast(s) : 0.f;    // tokens past the end carry no mass
        const float wm = mass ? w * mcur : w;           // ... and every token its own

        if (EPI == EPI_NONE || EPI == EPI_ACCUM_U) {
#pragma unroll
            for (int mb = 0; mb < RB; ++mb)
#pragma unroll
                for (int j = 0; j < 16; ++j) cs[mb][j] = fmaf(acc[mb][j], wm, cs[mb][j]);
        }

        if (EPI == EPI_ACCUM_U) {
            // Transpose the coupling tile (tokens in lanes -> tokens along K) through LDS as bf16.
            // With fp32 I/O the weights and the values are split into hi + lo parts (three products);
            // with bf16 I/O one product is enough: the rounding of the weights (2^-9, zero mean)
            // averages out over the tokens and stays far below the rounding of the bf16 output.
            constexpr bool kSplit = io_is_f32<IO>::value;
#pragma unroll
            for (int mb = 0; mb < RB; ++mb)
#pragma unroll
                for (int j = 0; j < 16; ++j) {
                    const float v = acc[mb][j] * wm;
                    const __bf16 h = (__bf16)v;
                    const int pv = pivot_of(mb, j, kg);
                    tr_hi[pv * kTrStride + i] = __builtin_bit_cast(uint16_t, h);
                    if (kSplit) tr_lo[pv * kTrStride + i] = __builtin_bit_cast(uint16_t, (__bf16)(v - (float)h));
                }
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
            for (int s = 0; s < 2; ++s) {
#pragma unroll
                for (int mb = 0; mb < RB; ++mb) {
                    const bf16x8 ah = *reinterpret_cast<const bf16x8*>(tr_hi + (32 * mb + i) * kTrStride + 16 * s + 8 * kg);
#pragma unroll
                    for (int nb = 0; nb < NB; ++nb)
                        U[mb][nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ah, vh[s][nb], U[mb][nb], 0, 0, 0);
                    if (kSplit) {
                        const bf16x8 al = *reinterpret_cast<const bf16x8*>(tr_lo + (32 * mb + i) * kTrStride + 16 * s + 8 * kg);
#pragma unroll
                        for (int nb = 0; nb < NB; ++nb) {
                            U[mb][nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(al, vh[s][nb], U[mb][nb], 0, 0, 0);
                            U[mb][nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ah, vl[s][nb], U[mb][nb], 0, 0, 0);
                        }
                    }
                }
            }
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
        }

        if (EPI == EPI_EXPAND) {
            f32x16 oacc[NB];
#pragma unroll
            for (int nb = 0; nb < NB; ++nb)
#pragma unroll
                for (int j = 0; j < 16; ++j) oacc[nb][j] = 0.f;
            constexpr bool kSplit = io_is_f32<IO>::value;   // see the accumulation pass
#pragma unroll
            for (int s = 0; s < 2 * RB; ++s) {
                f32x8 wv;
#pragma unroll
                for (int e = 0; e < 8; ++e) wv[e] = acc[s >> 1][8 * (s & 1) + e] * w;
                bf16x8 ah, al;
                if (kSplit) split_bf16(wv, ah, al);
                else ah = __builtin_convertvector(wv, bf16x8);
#pragma unroll
                for (int nb = 0; nb < NB; ++nb) {
                    const bf16x8 yh = yf_hi[(s * NB + nb) * 64 + lane];
                    oacc[nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ah, yh, oacc[nb], 0, 0, 0);
                    if (kSplit) {
                        const bf16x8 yl = yf_lo[(s * NB + nb) * 64 + lane];
                        oacc[nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(al, yh, oacc[nb], 0, 0, 0);
                        oacc[nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ah, yl, oacc[nb], 0, 0, 0);
                    }
                }
            }
            // one address per lane and tile; the row of accumulator register j is a compile-time offset
            const int row0 = tile * kTileTokens + 4 * kg;
            IO* const lane_base = out + ((size_t)g * stride + row0) * D;
            if ((tile + 1) * kTileTokens <= n) {   // whole tile in range: no per-row test
#pragma unroll
                for (int j = 0; j < 16; ++j)
                    store_out<NB>(lane_base + (8 * (j >> 2) + (j & 3)) * D, i, oacc[0][j], oacc[NB - 1][j]);
            } else {
#pragma unroll
                for (int j = 0; j < 16; ++j)
                    if (row0 + 8 * (j >> 2) + (j & 3) < n)
                        store_out<NB>(lane_base + (8 * (j >> 2) + (j & 3)) * D, i, oacc[0][j], oacc[NB - 1][j]);
            }
        }

        if (EPI == EPI_GAMMA) {
            // cs holds rho_t = beta_t / colsum_t in accumulator layout.  The addresses are built here,
            // per tile, from opaque copies of the sizes: hoisted out of the tile loop they would be 32
            // live 64-bit values, i.e. spills reloaded in front of every store.
            if (tok < n) {
                const int rr = opaque_scalar(p.r);
                const size_t nn = (size_t)opaque_scalar(n);
                if (side == 1) {
                    float* const row = p.gamma1 + ((size_t)g * nn + tok) * rr + 4 * kg;
                    const bool vec = (rr & 3) == 0;   // rows stay 16-byte aligned
#pragma unroll
                    for (int mb = 0; mb < RB; ++mb)
#pragma unroll
                        for (int q = 0; q < 4; ++q) {
                            const int pv0 = 32 * mb + 8 * q + 4 * kg;
                            f32x4 v;
#pragma unroll
                            for (int e = 0; e < 4; ++e) v[e] = acc[mb][4 * q + e] * wm * cs[mb][4 * q + e];
                            if (vec) {
                                if (pv0 < rr) *as_global(reinterpret_cast<f32x4*>(row + 32 * mb + 8 * q)) = v;
                            } else {
#pragma unroll
                                for (int e = 0; e < 4; ++e)
                                    if (pv0 + e < rr) as_global(row)[32 * mb + 8 * q + e] = v[e];
                            }
                        }
                } else {
                    float* const col = p.gamma2 + ((size_t)g * rr + 4 * kg) * nn + tok;
#pragma unroll
                    for (int mb = 0; mb < RB; ++mb)
#pragma unroll
                        for (int j = 0; j < 16; ++j) {
                            const int pc = 32 * mb + 8 * (j >> 2) + (j & 3);   // pivot minus 4 * kg
                            if (pc + 4 * kg < rr) as_global(col)[(size_t)pc * nn] = acc[mb][j] * wm * cs[mb][j];
                        }
                }
            }
        }
        xc = xn;
        mcur = mnext;
    }
    xfirst = xc;
    mfirst = mcur;
}

// A workgroup that leaves because a wait between workgroups gave up fills the rows it owns with NaN
// (the output rows of its query chunk, or its rows of the first coupling): whoever reads the result
// sees at once that the call failed, also without looking at the status words.
template <typename IO, int D>
__device__ __forceinline__ void poison_rows(const FusedParams& p, int g, int tile_begin, int tile_end, int threads)
{
    const int n = p.n_side[1];
    const int row0 = tile_begin * kTileTokens, row1 = min(n, tile_end * kTileTokens);
    if (row1 <= row0) return;
    const float nanf32 = __builtin_nanf("");
    if (p.out != nullptr) {
        IO* base = reinterpret_cast<IO*>(p.out) + ((size_t)g * p.stride_side[1] + row0) * D;
        const int count = (row1 - row0) * D;
        for (int e = threadIdx.x; e < count; e += threads) {
            if constexpr (io_is_f32<IO>::value) as_global(base)[e] = nanf32;
            else as_global(base)[e] = (uint16_t)0x7fc0u;
        }
    } else if (p.gamma1 != nullptr) {
        float* base = p.gamma1 + ((size_t)g * n + row0) * p.r;
        const int count = (row1 - row0) * p.r;
        for (int e = threadIdx.x; e < count; e += threads) as_global(base)[e] = nanf32;
    }
}

// ---------------------------------------------------------------------------------------------
// the kernel
// ---------------------------------------------------------------------------------------------
// A workgroup owns one chunk of tokens of one problem and runs BOTH solves on it, alternating
// key-side and query-side passes.  The cross-workgroup reduction of a pass is split in two: the
// partial column sums are posted right after the pass, and collected only when that side's next
// pass is about to start -- one whole pass of the other side later -- so the latency of the
// exchange (and the spread between workgroups) is hidden behind useful work.
template <typename IO, int D, int RB, int WAVES>
__global__ void __launch_bounds__(WAVES * 64, 2) lot_fused_kernel(FusedParams p)
{
    constexpr int NB = D / 32;
    constexpr int kThreads = WAVES * 64;
    __shared__ float s_wave_part[2][WAVES][64];   // per side: the reader of one pass never meets the writers of the next
    __shared__ float s_tot[2][64];     // cluster == 1: this workgroup's column sums, per side
    __shared__ float s_g[2][64];       // pivot potentials per side (0 = keys, 1 = queries)
    __shared__ float s_rho[2][64];     // beta_t / colsum_t after the last iteration
    __shared__ float s_csinv[64];      // 1 / colsum_t of the key side after the last iteration
    __shared__ float s_beta[64];
    __shared__ __attribute__((aligned(16))) float s_u[64 * D];
    __shared__ __attribute__((aligned(16))) uint16_t s_tr[WAVES * 2 * 64 * kTrStride];
    // the pivots' bf16 pieces for the similarity products where those are used (the tile loop reads them from here)
    __shared__ __attribute__((aligned(16))) char s_zf[similarity_by_pieces<IO, D, RB, WAVES>() ? PieceStashBytes<D, RB>::value : 16];
    __shared__ unsigned long long s_prev[2][2][64];   // last word seen per (side, parity, pivot)
    __shared__ int s_ok;
    __shared__ int s_okx[2];           // outcome of the collect inside an exchange, per side

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // uniform: tile indices and bases stay scalar
    const int i = lane & 31, kg = lane >> 5;
    const int r = p.r;
    const float c1 = kLog2e / p.eps;
    const int ntiles_side[2] = {(p.n_side[0] + kTileTokens - 1) / kTileTokens,
                                (p.n_side[1] + kTileTokens - 1) / kTileTokens};
    uint16_t* tr_hi = s_tr + (wave * 2 + 0) * 64 * kTrStride;
    uint16_t* tr_lo = s_tr + (wave * 2 + 1) * 64 * kTrStride;
    bf16x8* yf_hi = reinterpret_cast<bf16x8*>(s_tr);
    bf16x8* yf_lo = yf_hi + 2 * RB * NB * 64;
    const bool attention = p.mode == MODE_ATTENTION;

    for (int item = blockIdx.x; item < p.num_items; item += gridDim.x) {
        LOT_STAMP(0);
        const int g = item / p.cluster, chunk = item % p.cluster, h = g % p.H;
        const int tile_begins[2] = {chunk * p.tpw_side[0], chunk * p.tpw_side[1]};
        const int tile_ends[2] = {min(ntiles_side[0], tile_begins[0] + p.tpw_side[0]),
                                  min(ntiles_side[1], tile_begins[1] + p.tpw_side[1])};
        const float* beta = p.beta + (size_t)h * r;
        const IO* Xs[2] = {reinterpret_cast<const IO*>(p.K), reinterpret_cast<const IO*>(p.Q)};

        // the first key tile is requested before anything else: its latency overlaps the set-up
        Frag<IO, D> xfirst;
        float mfirst = 1.f;
        {
            const int tok = min((tile_begins[0] + wave) * kTileTokens + i, p.n_side[0] - 1);
            load_tokens<D>(xfirst, Xs[0] + ((size_t)g * p.stride_side[0] + tok) * D, kg);
            if (p.mass_side[0]) mfirst = (float)p.n_side[0] * as_global(p.mass_side[0])[(size_t)g * p.n_side[0] + tok];
        }
        // (beta is requested together with the pivots: one wait for both, not two round trips)
        const float beta_read = as_global(beta)[min(tid & 63, r - 1)];   // unconditional: issued with the loads around it
        Frag<IO, D> zf[RB];
#pragma unroll
        for (int mb = 0; mb < RB; ++mb) {
            const int t = 32 * mb + i;
            load_pivots<D>(zf[mb], p.Z + ((size_t)h * r + min(t, r - 1)) * D, kg, t < r);
        }
        if constexpr (similarity_by_pieces<IO, D, RB, WAVES>()) {
            if (wave == 0) stash_pivot_pieces<D, RB>(s_zf, zf, lane);
        }
        if (tid < 128) s_g[tid >> 6][tid & 63] = (tid & 63) < r ? 0.f : kNegBig;
        if (tid < 64) s_beta[tid] = tid < r ? beta_read : 1.f;
        if (tid < 256) (&s_prev[0][0][0])[tid] = 0ull;   // the accumulators start at zero in every launch
        if (blockIdx.x == 0 && tid == 0 && item == (int)blockIdx.x)
            __hip_atomic_store(p.status + 1, p.nonce, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);   // this launch; nobody else writes it
        if (p.cluster > 1 && chunk == 0) {
            // The first workgroup of a problem zeroes the problem's accumulators and counters, then
            // publishes this launch's nonce; the cluster waits for it before its first post.  (No
            // separate clearing kernel: one launch per call.)
            if (tid < 256) __hip_atomic_store(p.colacc + (size_t)g * 256 + tid, 0ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            if (tid == 0) {
                __hip_atomic_store(p.arrive + g, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                __hip_atomic_store(p.yready + g, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
            publish_barrier();   // the zeroes have been acknowledged
            if (tid == 0) __hip_atomic_store(p.cleared + g, p.nonce, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        lds_barrier();
        f32x16 cs[RB], U[RB][NB];
        LOT_STAMP(1);

        unsigned long long early_word = 0, early_word2 = 0;   // wavefront 0: polls issued ahead of their use
#ifdef LOT_TRACE
        unsigned long long repolls = 0, valid_a = 0;
#endif

        // ---- wavefront 0: take the column sums of pass `it` of `side` (lane = pivot) and apply the
        //      pivot-side update.  No barrier inside; the caller publishes the result.
        auto collect_w0 = [&](int side, int it, bool final, unsigned long long early) -> bool {
            const int ln = fresh_lane();
            const int rr = opaque_scalar(r);
            float tot = 0.f;
            bool ok = true;
            if (p.cluster > 1) {
                // every pivot's word carries its own arrival count: complete when all 64 agree
                const unsigned long long* src = p.colacc + (((size_t)2 * g + side) * 2 + (it & 1)) * 64 + ln;
                const unsigned long long prev = s_prev[side][it & 1][ln];
                unsigned long long word = early;   // a poll that was started ahead; validated here
                ok = __all(((unsigned)((word >> 56) - (prev >> 56)) & 0xffu) == (unsigned)p.cluster);
#ifdef LOT_TRACE
                valid_a += ok ? 1 : 0;
#endif
                for (uint32_t k = 0; !ok && k < p.spin_limit; ++k) {
#ifdef LOT_TRACE
                    ++repolls;
#endif
                    word = __hip_atomic_load(src, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    if (__all(((unsigned)((word >> 56) - (prev >> 56)) & 0xffu) == (unsigned)p.cluster)) { ok = true; break; }
                    if ((k & 63u) == 63u && gave_up(p.status, p.nonce)) break;
                    __builtin_amdgcn_s_sleep(1);
                }
                s_prev[side][it & 1][ln] = word;
                const unsigned long long mask = (1ull << 56) - 1ull;
                tot = (float)(long long)((word & mask) - (prev & mask)) * p.fx_unscale;
                if (!ok && ln == 0) give_up(p.status, p.nonce);
            } else {
                tot = s_tot[side][ln];
            }
            if (ln < rr) {
                // (sums exchanged in fixed point: one below the resolution reads as half a unit)
                const float c = fmaxf(tot, p.cluster > 1 ? 0.5f * p.fx_unscale : 1.0e-37f);
                const float b = s_beta[ln];
                if (!final) {
                    s_g[side][ln] += p.eps * logf((float)opaque_scalar(p.n_side[side]) * b / c);
                } else {
                    // the last pass's potentials stay: the epilogue rebuilds its coupling from them
                    s_rho[side][ln] = b / c;
                    if (side == 0) s_csinv[ln] = 1.f / c;
                }
            } else if (final) {
                s_rho[side][ln] = 0.f;
                if (side == 0) s_csinv[ln] = 0.f;
            }
            return ok;
        };

        // ---- after a pass: post this workgroup's share (column sums; U on the last key pass) and,
        //      in the same breath, collect the other side's previous pass, which was posted one
        //      whole pass ago.  One workgroup barrier in all (more when U is reduced).
        auto exchange = [&](int side, int it, bool with_u, int cside, int cit, bool cfinal) -> bool {
            if (p.cluster > 1 && it == 1 && side == 0) {
                // first post of this launch: the problem's accumulators must have been zeroed
                if (tid == 0) {
                    bool ok = false;
                    for (uint32_t k = 0; k < p.spin_limit; ++k) {
                        if (__hip_atomic_load(p.cleared + g, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == p.nonce) { ok = true; break; }
                        __builtin_amdgcn_s_sleep(1);
                    }
                    if (!ok) give_up(p.status, p.nonce);
                    s_ok = ok;
                }
                lds_barrier();
                if (!s_ok) return false;
            }
            LOT_STAMP(9 + 6 * ((it - 1) * 2 + side));   // pass done
            __builtin_amdgcn_s_setprio(3);
            if (p.cluster > 1 && wave == 0 && cit >= 1) {
                // start the poll now; it completes while this pass's sums are reduced
                early_word = ldc_u64(coherent_view(p.colacc),
                                     (uint32_t)(((((size_t)2 * g + cside) * 2 + (cit & 1)) * 64 + lane) * 8));
                // after the very last pass the query side is collected as well
                if (side == 1 && it == p.iters)
                    early_word2 = ldc_u64(coherent_view(p.colacc),
                                          (uint32_t)(((((size_t)2 * g + 1) * 2 + (it & 1)) * 64 + lane) * 8));
            }
            {
                // this wavefront's column sums: one pivot per lane after the transposing reduction
                float c[16 * RB];
#pragma unroll
                for (int mb = 0; mb < RB; ++mb)
#pragma unroll
                    for (int j = 0; j < 16; ++j) c[16 * mb + j] = cs[mb][j];
                const float total = reduce_scatter_tokens<16 * RB>(c, i);
                const int q = RB == 2 ? i : i >> 1;   // accumulator register this lane ended up with
                s_wave_part[side][wave][32 * (q >> 4) + 8 * ((q & 15) >> 2) + 4 * kg + (q & 3)] = total;
            }
            LOT_STAMP(10 + 6 * ((it - 1) * 2 + side));   // own sums reduced
            if (wave == 0) {
                // The other side's sums do not depend on this pass at all: they are taken now, while
                // the slower wavefronts are still arriving, and the updated potentials are published
                // by the barrier below.
                bool ok = true;
                if (cit >= 1) ok = collect_w0(cside, cit, cfinal, early_word);
                if (fresh_lane() == 0) s_okx[side] = ok;
            }
            LOT_STAMP(11 + 6 * ((it - 1) * 2 + side));   // collected
            if (with_u) {
                // Workgroup total of U in s_u.  The wavefronts dump their accumulators into separate
                // buffers (s_u itself and the now idle transposition area), in rounds when there are
                // more wavefronts than buffers; then every thread sums its elements over the buffers.
                // The order of the additions is fixed.
                constexpr int kElems = 64 * D;
                constexpr int kExtra = (int)(sizeof(s_tr) / (kElems * sizeof(float)));
                constexpr int kBufs = WAVES < 1 + kExtra ? WAVES : 1 + kExtra;
                float* const extra = reinterpret_cast<float*>(s_tr);
                lds_barrier();   // every wavefront has finished its transpositions: the area is free
                for (int round = 0; round * kBufs < WAVES; ++round) {
                    if (wave / kBufs == round) {
                        const int b = wave % kBufs;
                        float* const buf = b == 0 ? s_u : extra + (b - 1) * kElems;
#pragma unroll
                        for (int mb = 0; mb < RB; ++mb)
#pragma unroll
                            for (int nb = 0; nb < NB; ++nb)
#pragma unroll
                                for (int j = 0; j < 16; ++j) {
                                    float* dst = &buf[pivot_of(mb, j, kg) * D + NB * i + nb];
                                    *dst = round == 0 ? U[mb][nb][j] : *dst + U[mb][nb][j];
                                }
                    }
                    lds_barrier();
                }
                for (int e = wave * 64 + fresh_lane(); e < kElems; e += kThreads) {
                    float acc = s_u[e];
#pragma unroll
                    for (int b = 1; b < kBufs; ++b) acc += extra[(b - 1) * kElems + e];
                    s_u[e] = acc;
                }
                lds_barrier();
            } else {
                lds_barrier();
            }
            LOT_STAMP(12 + 6 * ((it - 1) * 2 + side));   // all wavefronts' sums in LDS, potentials published
            if (wave == 0) {
                const int ln = fresh_lane();
                float tot = s_wave_part[side][0][ln];
#pragma unroll
                for (int wv = 1; wv < WAVES; ++wv) tot += s_wave_part[side][wv][ln];
                if (ln >= opaque_scalar(r)) tot = 0.f;   // padding pivots (their LDS slots may never have been written)
                if (p.cluster > 1) {
                    // one fire-and-forget atomic per pivot: the workgroup's column sum in fixed point
                    // (integer addition: the total does not depend on arrival order) plus one count
                    const unsigned long long word = (1ull << 56) + (unsigned long long)__float2ll_rn(tot * p.fx_scale);
                    __hip_atomic_fetch_add(p.colacc + (((size_t)2 * g + side) * 2 + (it & 1)) * 64 + ln, word,
                                           __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                } else {
                    s_tot[side][ln] = tot;
                }
                LOT_STAMP(13 + 6 * ((it - 1) * 2 + side));   // posted
            }
            if (p.cluster > 1 && with_u) {
                float* up = p.u_part + ((size_t)g * p.cluster_cap + chunk) * 64 * D;
                for (int e = wave * 64 + fresh_lane(); e < 64 * D; e += kThreads) st_coherent(up + e, s_u[e]);
                publish_barrier();   // the stores above have been acknowledged
                if (tid == 0) __hip_atomic_fetch_add(p.arrive + g, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
            __builtin_amdgcn_s_setprio(0);
            return s_okx[side] != 0;
        };

        for (int it = 1; it <= p.iters; ++it) {
            for (int side = 0; side < 2; ++side) {
                // the pass after this one: the other side, except that the last query pass is
                // followed by an epilogue pass (queries again for attention, keys for couplings)
                const int next_side = (side == 1 && it == p.iters) ? (attention ? 1 : 0) : (side ^ 1);
                const IO* Xnext = Xs[next_side];
#pragma unroll
                for (int mb = 0; mb < RB; ++mb)
#pragma unroll
                    for (int j = 0; j < 16; ++j) cs[mb][j] = 0.f;
                const bool with_u = attention && side == 0 && it == p.iters;
                LOT_STAMP(8 + 6 * ((it - 1) * 2 + side));   // pass starts
                if (with_u) {
#pragma unroll
                    for (int mb = 0; mb < RB; ++mb)
#pragma unroll
                        for (int nb = 0; nb < NB; ++nb)
#pragma unroll
                            for (int j = 0; j < 16; ++j) U[mb][nb][j] = 0.f;
                    run_pass<IO, D, RB, EPI_ACCUM_U, WAVES>(p, Xs[side], Xnext, next_side, xfirst, mfirst, g, side, tile_begins, tile_ends[side], lane, wave, c1, zf, s_zf, s_g[side], cs,
                                                     reinterpret_cast<const IO*>(p.V), U, tr_hi, tr_lo, yf_hi, yf_lo, nullptr);
                } else {
                    run_pass<IO, D, RB, EPI_NONE, WAVES>(p, Xs[side], Xnext, next_side, xfirst, mfirst, g, side, tile_begins, tile_ends[side], lane, wave, c1, zf, s_zf, s_g[side], cs,
                                                  nullptr, U, tr_hi, tr_lo, yf_hi, yf_lo, nullptr);
                }
                // what is collected along with this post: keys' pass `it` after a query pass (for
                // the last iteration that is the keys' final update), queries' pass `it - 1` after
                // a key pass
                if (!exchange(side, it, with_u, side ^ 1, side == 1 ? it : it - 1, side == 1 && it == p.iters)) {
                    poison_rows<IO, D>(p, g, tile_begins[1], tile_ends[1], kThreads);
                    return;
                }
            }
        }
        float* yt = p.y_tile + (size_t)g * 64 * D;
        if (attention && p.cluster > 1) {
            // The U partials were posted a whole pass ago.  Each workgroup of the cluster sums one
            // slice of them (raw, still unnormalised) and publishes it; this runs before the last
            // column sums are collected, whose polls are already in flight.
            __builtin_amdgcn_s_setprio(3);
            if (tid == 0) {
                const bool ok = spin_until(p.arrive + g, (uint32_t)p.cluster, p.status, p.nonce, p.spin_limit);
                if (!ok) give_up(p.status, p.nonce);
                s_ok = ok;
            }
            lds_barrier();
            if (!s_ok) { poison_rows<IO, D>(p, g, tile_begins[1], tile_ends[1], kThreads); return; }
            const int per = (64 * D + p.cluster - 1) / p.cluster;
            const int e0 = chunk * per, e1 = min(64 * D, e0 + per);
            const float* up = p.u_part + (size_t)g * p.cluster_cap * 64 * D;
            const __amdgpu_buffer_rsrc_t upv = coherent_view(up);
            for (int e = e0 + wave * 64 + fresh_lane(); e < e1; e += kThreads) {
                float acc = 0.f;
                for (int k0 = 0; k0 < p.cluster; k0 += 8) {
                    float v[8];
#pragma unroll
                    for (int j = 0; j < 8; ++j)
                        v[j] = ldc_f32(upv, (uint32_t)(((size_t)min(k0 + j, p.cluster - 1) * 64 * D + e) * 4));
#pragma unroll
                    for (int j = 0; j < 8; ++j) acc += (k0 + j < p.cluster) ? v[j] : 0.f;
                }
                st_coherent(yt + e, acc);
            }
            publish_barrier();   // the slice has been acknowledged
            if (tid == 0) __hip_atomic_fetch_add(p.yready + g, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            __builtin_amdgcn_s_setprio(0);
        }
        // the queries' final update (the keys' was taken with the last exchange)
        __builtin_amdgcn_s_setprio(3);
        if (wave == 0) {
            const bool ok = collect_w0(1, p.iters, true, early_word2);
            if (lane == 0) s_ok = ok;
        }
        lds_barrier();
        __builtin_amdgcn_s_setprio(0);
        if (!s_ok) { poison_rows<IO, D>(p, g, tile_begins[1], tile_ends[1], kThreads); return; }

        LOT_STAMP(2);
        if (!attention) {
            for (int side = 0; side < 2; ++side) {
                load_pivot_vector<RB>(cs, s_rho[side], kg);
                run_pass<IO, D, RB, EPI_GAMMA, WAVES>(p, Xs[side], side == 0 ? Xs[1] : nullptr, 1, xfirst, mfirst, g, side, tile_begins, tile_ends[side], lane, wave, c1, zf, s_zf, s_g[side], cs,
                                               nullptr, U, tr_hi, tr_lo, yf_hi, yf_lo, nullptr);
            }
        } else {
            // Y''_t = n * rho1_t * U_t / colsum2_t  ->  s_u
            if (p.cluster == 1) {
                for (int e = wave * 64 + fresh_lane(); e < 64 * D; e += kThreads) s_u[e] *= s_csinv[e / D] * ((float)p.n_side[1] * s_rho[1][e / D]);
            } else {
                __builtin_amdgcn_s_setprio(3);
                if (tid == 0) {
                    const bool ok = spin_until(p.yready + g, (uint32_t)p.cluster, p.status, p.nonce, p.spin_limit);
                    if (!ok) give_up(p.status, p.nonce);
                    s_ok = ok;
                }
                lds_barrier();
                if (!s_ok) { poison_rows<IO, D>(p, g, tile_begins[1], tile_ends[1], kThreads); return; }
                constexpr int kChunks = 64 * D / 4 / kThreads;   // 16-byte chunks per thread
                const int ft = wave * 64 + fresh_lane();
                f32x4 v[kChunks];
                const __amdgpu_buffer_rsrc_t ytv = coherent_view(yt);
#pragma unroll
                for (int j = 0; j < kChunks; ++j) v[j] = ldc_f32x4(ytv, (uint32_t)(16 * (ft + j * kThreads)));
#pragma unroll
                for (int j = 0; j < kChunks; ++j) {
                    const int e = 4 * (ft + j * kThreads);
                    const float sc = s_csinv[e / D] * ((float)p.n_side[1] * s_rho[1][e / D]);
#pragma unroll
                    for (int c = 0; c < 4; ++c) s_u[e + c] = v[j][c] * sc;
                }
                __builtin_amdgcn_s_setprio(0);
            }
            lds_barrier();
            // lay Y'' out as MFMA B fragments (bf16 hi + lo)
            LOT_STAMP(3);
            for (int f = wave * 64 + fresh_lane(); f < 2 * RB * NB * 64; f += kThreads) {
                const int fl = f & 63, fi = fl & 31, fkg = fl >> 5;
                const int snb = f >> 6, s = snb / NB, nb = snb % NB;
                f32x8 t;
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const int pv = 32 * (s >> 1) + 16 * (s & 1) + 8 * (e >> 2) + 4 * fkg + (e & 3);
                    t[e] = s_u[pv * D + NB * fi + nb];
                }
                bf16x8 hi, lo;
                split_bf16(t, hi, lo);
                yf_hi[f] = hi;
                yf_lo[f] = lo;
            }
            lds_barrier();
            LOT_STAMP(4);
            run_pass<IO, D, RB, EPI_EXPAND, WAVES>(p, Xs[1], nullptr, 1, xfirst, mfirst, g, 1, tile_begins, tile_ends[1], lane, wave, c1, zf, s_zf, s_g[1], cs,
                                            nullptr, U, tr_hi, tr_lo, yf_hi, yf_lo, reinterpret_cast<IO*>(p.out));
        }
        LOT_STAMP(5);
#ifdef LOT_TRACE
        if (threadIdx.x == 0 && p.trace) p.trace[(size_t)blockIdx.x * 128 + 6] = repolls;
        if (threadIdx.x == 0 && p.trace) p.trace[(size_t)blockIdx.x * 128 + 7] = valid_a;
#endif
        __syncthreads();   // LDS is reused by the next item
    }
}

template <typename IO, int D, int RB, int WAVES>
int launch(const Args& a, bool want_out)
{
    constexpr int kThreads = WAVES * 64;
    const lot_shape& s = a.s;
    const int G = s.B * s.H;
    auto kernel = lot_fused_kernel<IO, D, RB, WAVES>;

    static thread_local int capacity_cache[8] = {0};   // per device ordinal
    int dev = 0;
    LOT_HIP_CHECK(hipGetDevice(&dev));
    int capacity = (dev >= 0 && dev < 8) ? capacity_cache[dev] : 0;
    if (capacity == 0) {
        int per_cu = 0, cus = 0;
        LOT_HIP_CHECK(hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, kernel, kThreads, 0));
        LOT_HIP_CHECK(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev));
        capacity = per_cu * cus;
        if (capacity < 1) { last_hip_error() = hipErrorLaunchOutOfResources; return LOT_ERR_HIP; }
        if (capacity > max_resident_wgs()) capacity = max_resident_wgs();
        if (dev >= 0 && dev < 8) capacity_cache[dev] = capacity;
    }

    // per side: 0 = keys and values, 1 = queries; equal unless this is cross attention
    const int n_side[2] = {a.n_k > 0 ? a.n_k : s.n, a.n_q > 0 ? a.n_q : s.n};
    const int nt_side[2] = {(n_side[0] + kTileTokens - 1) / kTileTokens, (n_side[1] + kTileTokens - 1) / kTileTokens};
    const int ntiles = nt_side[0] > nt_side[1] ? nt_side[0] : nt_side[1];
    int cluster = fused_cluster_bound(s);
    {
        const int by_tiles = (ntiles + WAVES - 1) / WAVES;   // at least one tile per wavefront
        if (cluster > by_tiles) cluster = by_tiles;
    }
    if (cluster > capacity / G) cluster = capacity / G;
    if (cluster < 1) cluster = 1;
    const int tiles_per_wg = (ntiles + cluster - 1) / cluster;
    cluster = (ntiles + tiles_per_wg - 1) / tiles_per_wg;

    FusedParams p{};
    p.Q = a.Q; p.K = a.K; p.V = a.V; p.Z = a.Z; p.beta = a.beta; p.out = a.out;
    p.gamma1 = a.gamma1; p.gamma2 = a.gamma2;
    p.status = (unsigned long long*)(a.ws + a.lay.status);
    p.arrive = (uint32_t*)(a.ws + a.lay.counters);
    p.yready = p.arrive + G;
    p.cleared = (unsigned long long*)(a.ws + a.lay.cleared);
    p.colacc = (unsigned long long*)(a.ws + a.lay.colacc);
    p.u_part = (float*)(a.ws + a.lay.u_part);
    p.y_tile = (float*)(a.ws + a.lay.y_tile);
    p.G = G; p.H = s.H; p.r = s.r;
    for (int sd = 0; sd < 2; ++sd) {
        p.n_side[sd] = n_side[sd];
        p.stride_side[sd] = a.n_stride > 0 ? a.n_stride : n_side[sd];
        p.tpw_side[sd] = (nt_side[sd] + cluster - 1) / cluster;
    }
    p.mass_side[0] = a.mass_k; p.mass_side[1] = a.mass_q;
    p.cluster = cluster; p.cluster_cap = fused_cluster_bound(s);
    p.num_items = G * cluster; p.iters = a.iters; p.mode = want_out ? MODE_ATTENTION : MODE_COUPLINGS;
    p.eps = a.eps;
    p.spin_limit = spin_limit();
    // only where the last 8 MiB of the workspace lie wholly inside the reference path's regions
    p.trace = a.lay.total >= a.lay.C + (8u << 20) ? (unsigned long long*)(a.ws + a.lay.total - (8u << 20)) : nullptr;

    // fixed-point format of the exchanged column sums
    {
        const int frac = fused_exchange_frac_bits(n_side[0] > n_side[1] ? n_side[0] : n_side[1], a.iters);
        if (frac < 0) return LOT_ERR_PATH;
        p.fx_scale = std::ldexp(1.0f, frac);
        p.fx_unscale = std::ldexp(1.0f, -frac);
    }

    // A value that no earlier launch has used: the kernel's own clearing of its counters is
    // published under it, and so is a wait that gives up.
    p.nonce = next_nonce();

    const int grid = p.num_items < capacity ? p.num_items : capacity;
    // An ordinary launch: the grid never exceeds the number of workgroups the device can hold at
    // once (occupancy query above), which is what the cross-workgroup waits need, and the waits are
    // bounded in any case.  (A cooperative launch would assert the same thing, but kernel tracing
    // tools do not survive it.)
    kernel<<<dim3(grid), dim3(kThreads), 0, a.stream>>>(p);
    LOT_HIP_CHECK(hipGetLastError());
    return LOT_OK;
}

// Workgroup size: eight wavefronts (one workgroup per compute unit) when the problems fit one
// round of such workgroups -- fewer, larger workgroups mean fewer participants per exchange and a
// shorter dispatch ramp; four wavefronts (two workgroups per compute unit) otherwise, which keeps
// twice as many work items resident.
template <typename IO, int D, int RB>
int launch_sized(const Args& a, bool want_out)
{
    int dev = 0, cus = 0;
    LOT_HIP_CHECK(hipGetDevice(&dev));
    LOT_HIP_CHECK(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev));
    // (fp32 I/O at d = 64 with two pivot blocks: the 24 KB of pivot pieces leave no room in the LDS for
    // two workgroups per compute unit, so that variant always runs with eight wavefronts)
    if constexpr (io_is_f32<IO>::value && D == 64 && RB == 2) {
        return launch<IO, D, RB, 8>(a, want_out);
    } else {
        if (a.s.B * a.s.H <= cus) return launch<IO, D, RB, 8>(a, want_out);
        return launch<IO, D, RB, 4>(a, want_out);
    }
}

template <typename IO>
int dispatch(const Args& a, bool want_out)
{
    const int d = a.s.d_k, rb = a.s.r <= 32 ? 1 : 2;
    if (d == 32 && rb == 1) return launch_sized<IO, 32, 1>(a, want_out);
    if (d == 32 && rb == 2) return launch_sized<IO, 32, 2>(a, want_out);
    if (d == 64 && rb == 1) return launch_sized<IO, 64, 1>(a, want_out);
    if (d == 64 && rb == 2) return launch_sized<IO, 64, 2>(a, want_out);
    return LOT_ERR_PATH;
}

}  // namespace

int run_fused(const Args& a, bool want_out)
{
    if (!fused_supports(a.s)) return LOT_ERR_PATH;
    return a.s.io_dtype == LOT_BF16 ? dispatch<uint16_t>(a, want_out) : dispatch<float>(a, want_out);
}

}  // namespace lot
