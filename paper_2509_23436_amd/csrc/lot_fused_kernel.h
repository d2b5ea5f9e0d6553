// The fused kernel of libLOT and its launcher, shared by the translation units that instantiate it
// (lot_fused.hip: the streaming variants; lot_fused_res.hip: the variants that keep the kernel matrix
// on chip).  See lot_fused.hip for the description of the work decomposition.
#pragma once
#ifndef LOT_ACCUM_AHEAD
#define LOT_ACCUM_AHEAD 3
#endif
#include <cmath>
#include <type_traits>

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
#ifndef LOT_TRACE_THREAD
#define LOT_TRACE_THREAD 0
#endif
#define LOT_STAMP(slot) do { if (threadIdx.x == LOT_TRACE_THREAD && (slot) < 128 && p.trace) p.trace[(size_t)blockIdx.x * 128 + (slot)] = wall_clock64(); } while (0)
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
    unsigned long long* colacc;   // [G][2 sides][2 parities][64]: count << kCountShift | fixed-point column sum
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
    float drift_half;            // NT > 0: a pivot's potential may move this many binary orders away from pivot 0's before the kernel matrix is recomputed
    unsigned long long* trace;   // LOT_TRACE builds only
};

// Format of an exchanged column sum: arrivals in the top ten bits (every wavefront but the first of every
// workgroup of a problem posts: up to 64 * 7), the fixed-point sum below.
constexpr int kCountShift = 54;
constexpr unsigned kCountMask = 0x3ffu;




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

// ---------------------------------------------------------------------------------------------
// on-chip kernel matrix ("resident" variants, NT > 0)
// ---------------------------------------------------------------------------------------------
// The scaling form of the iteration (paper, "Conditional OT": Gamma = Diag(u) exp(C/eps) Diag(v)) needs
// the kernel matrix exp(C/eps) only once: every later iteration is a matrix-vector product with it in
// each direction.  When a workgroup's share of that matrix fits on chip, the first pass of a side
// ("fill") computes  Kt_it = exp((C_it + gref_t - m_i)/eps)  (m_i the row maximum, gref the pivot
// potentials of that moment: zero in the first iteration) and keeps it -- the queries' share in
// registers, the keys' share in LDS -- and the following passes ("cheap") read neither Q nor K again
// and evaluate no exponential:
//     v_t = exp((g_t - gref_t)/eps - shift),  s_i = sum_t Kt_it v_t,  colsum_t = v_t sum_i Kt_it / s_i
// which are the same row-normalised couplings and column sums as a pass that recomputes everything
// (the shift and the row factors cancel).  The potentials may drift from gref by at most kDriftLimit
// binary orders between the largest and the smallest change (lot_debug_set can lower that for tests); beyond that (extreme eps) the next pass of
// that side is a fill again, with the current potentials folded in, so the result never depends on
// products that underflow.  With bf16 I/O the kept matrix is bf16 (pairs in one register): it meets the
// bf16 operands of the matrix instructions in the two contractions anyway, and a relative 2^-9 on a
// kernel entry is a change of eps 2^-9 in a similarity, below the rounding of the bf16 Q and K
// themselves; with fp32 I/O it is kept in fp32.
constexpr float kDriftLimit = 32.f;

typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
template <typename IO> struct res_packed { static constexpr bool value = !io_is_f32<IO>::value; };
// registers (or LDS words) per lane and tile
template <typename IO, int RB> struct ResWords { static constexpr int value = res_packed<IO>::value ? 8 * RB : 16 * RB; };

template <typename IO, int RB>
__device__ __forceinline__ void res_pack(uint32_t (&w)[(ResWords<IO, RB>::value)], const f32x16 (&e)[RB])
{
#pragma unroll
    for (int mb = 0; mb < RB; ++mb) {
        if constexpr (res_packed<IO>::value) {
#pragma unroll
            for (int q = 0; q < 8; ++q) {
                f32x2 pr;
                pr[0] = e[mb][2 * q];
                pr[1] = e[mb][2 * q + 1];
                w[8 * mb + q] = __builtin_bit_cast(uint32_t, __builtin_convertvector(pr, bf16x2));
            }
        } else {
#pragma unroll
            for (int j = 0; j < 16; ++j) {
                const float x = e[mb][j];   // (a scalar copy first: a bit cast of the vector element in place reads element 0)
                w[16 * mb + j] = __builtin_bit_cast(uint32_t, x);
            }
        }
    }
}
template <typename IO, int RB>
__device__ __forceinline__ void res_unpack(f32x16 (&e)[RB], const uint32_t (&w)[(ResWords<IO, RB>::value)])
{
#pragma unroll
    for (int mb = 0; mb < RB; ++mb) {
        if constexpr (res_packed<IO>::value) {
#pragma unroll
            for (int q = 0; q < 8; ++q) {
                e[mb][2 * q] = __builtin_bit_cast(float, w[8 * mb + q] << 16);
                e[mb][2 * q + 1] = __builtin_bit_cast(float, w[8 * mb + q] & 0xffff0000u);
            }
        } else {
#pragma unroll
            for (int j = 0; j < 16; ++j) e[mb][j] = __builtin_bit_cast(float, w[16 * mb + j]);
        }
    }
}
// the keys' share in LDS: 16-byte units [unit][lane] per (wavefront, tile slot)
template <int NW>
__device__ __forceinline__ void res_to_lds(u32x4* dst, const uint32_t (&w)[NW], int lane)
{
#pragma unroll
    for (int u = 0; u < NW / 4; ++u) {
        u32x4 t;
#pragma unroll
        for (int e = 0; e < 4; ++e) t[e] = w[4 * u + e];
        dst[u * 64 + lane] = t;
    }
}
template <int NW>
__device__ __forceinline__ void res_from_lds(uint32_t (&w)[NW], const u32x4* src, int lane)
{
#pragma unroll
    for (int u = 0; u < NW / 4; ++u) {
        const u32x4 t = src[u * 64 + lane];
#pragma unroll
        for (int e = 0; e < 4; ++e) w[4 * u + e] = t[e];
    }
}

// Request the rows of this wavefront's first tile of `side` (what a streaming pass expects in xfirst).
template <typename IO, int D>
__device__ __forceinline__ void request_first_tile(const FusedParams& p, const IO* X, Frag<IO, D>& xfirst,
                                                   int g, int side, int tile_begin, int lane, int wave)
{
    const int i = lane & 31, kg = lane >> 5;
    const int nn = p.n_side[side];
    const int tok = min((tile_begin + wave) * kTileTokens + i, nn - 1);
    load_tokens<D>(xfirst, X + ((size_t)g * p.stride_side[side] + tok) * D, kg);
}

// A pass that streams this wavefront's tiles of `side`, computes the kernel matrix like
// run_pass<EPI_NONE> (current potentials folded in, rows shifted by their maxima) and keeps it: in kq
// (registers) or, TO_LDS, in this wavefront's block of the LDS area.  It forms no sums: the caller
// follows it with a pass over the kept matrix with v = 1 (holding the column-sum accumulators as
// well would not leave the registers for it).  At most NT tiles per
// wavefront (the launcher's condition for these variants).  The loop over the slots is unrolled only
// where the slot picks registers.
template <typename IO, int D, int RB, int WAVES, int NT, bool TO_LDS>
__device__ __forceinline__ void fill_pass(
    const FusedParams& p, const IO* __restrict__ X, const IO* __restrict__ Xnext, int next_side,
    Frag<IO, D>& xfirst, int g, int side, const int (&tile_begins)[2], int tile_end, int lane, int wave, float c1,
    const void* zlds, const float* glds,
    uint32_t (&kq)[NT][(ResWords<IO, RB>::value)], u32x4* kres_wave)
{
    constexpr int NW = ResWords<IO, RB>::value;
    // the pivots come from LDS (bf16 operand fragments, or the bf16 pieces of fp32 pivots): held in
    // registers for the whole kernel they would crowd out the kept kernel matrix
    Frag<IO, D> zf[RB];
    if constexpr (!similarity_by_pieces<IO, D, RB, WAVES>()) {
        int zskew = 0;
        asm volatile("" : "+v"(zskew));
        fetch_pivots<D, RB>(zf, zlds, lane, zskew);
    }
    const int i = lane & 31, kg = lane >> 5;
    const int n = p.n_side[side];
    const int stride = p.stride_side[side];
    const int tile_begin = tile_begins[side];
    if (tile_begin + wave >= tile_end) {
        if (Xnext != nullptr) request_first_tile<IO, D>(p, Xnext, xfirst, g, next_side, tile_begins[next_side], lane, wave);
        return;
    }
    Frag<IO, D> xc = xfirst;
    constexpr int kUnrollSlots = TO_LDS ? 1 : NT;   // unrolled only where the slot picks registers
#pragma unroll kUnrollSlots
    for (int slot = 0; slot < NT; ++slot) {
        const int tile = tile_begin + wave + slot * WAVES;
        if (tile < tile_end) {
            Frag<IO, D> xn = xc;
            if (tile + WAVES < tile_end) {
                const int tok = min((tile + WAVES) * kTileTokens + i, n - 1);
                load_tokens<D>(xn, X + ((size_t)g * stride + tok) * D, kg);
            } else if (Xnext != nullptr) {
                request_first_tile<IO, D>(p, Xnext, xn, g, next_side, tile_begins[next_side], lane, wave);
            }
            int skew = 0;
            asm volatile("" : "+v"(skew));
            f32x16 acc[RB];
            load_pivot_vector<RB>(acc, glds + skew, kg);
            if constexpr (similarity_by_pieces<IO, D, RB, WAVES>()) similarity_pieces<D, RB>(acc, zlds, xc, lane, skew);
            else similarity<D, RB>(acc, zf, xc);

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
#pragma unroll
            for (int mb = 0; mb < RB; ++mb)
#pragma unroll
                for (int j = 0; j < 16; ++j) acc[mb][j] = exp2_fast(fmaf(acc[mb][j], c1, -mc));
            if constexpr (TO_LDS) {
                uint32_t packed[NW];
                res_pack<IO, RB>(packed, acc);
                res_to_lds<NW>(kres_wave + slot * (NW / 4) * 64, packed, lane);
            } else {
                res_pack<IO, RB>(kq[slot], acc);
            }
            xc = xn;
        }
    }
    xfirst = xc;
}

// The same pass for wavefronts that have a SIMD, and with it 512 registers, to themselves (four
// wavefronts per workgroup): nobody else is there to run while one waits for memory, so the rows of
// AHEAD tiles are kept in flight; the loop over the slots is unrolled for both sides.
template <typename IO, int D, int RB, int WAVES, int NT, bool TO_LDS, int AHEAD>
__device__ __forceinline__ void fill_pass_ahead(
    const FusedParams& p, const IO* __restrict__ X, const IO* __restrict__ Xnext, int next_side,
    Frag<IO, D>& xfirst, int g, int side, const int (&tile_begins)[2], int tile_end, int lane, int wave, float c1,
    const void* zlds, const float* glds,
    uint32_t (&kq)[NT][(ResWords<IO, RB>::value)], u32x4* kres_wave)
{
    constexpr int NW = ResWords<IO, RB>::value;
    Frag<IO, D> zf[RB];
    if constexpr (!similarity_by_pieces<IO, D, RB, WAVES>()) {
        int zskew = 0;
        asm volatile("" : "+v"(zskew));
        fetch_pivots<D, RB>(zf, zlds, lane, zskew);
    }
    int io = lane & 31;
    asm volatile("" : "+v"(io));     // (opaque: the addresses of all slots are not to be hoisted out of the iteration loop)
    const int kg = lane >> 5;
    const int n = p.n_side[side];
    const int stride = p.stride_side[side];
    const int tile_begin = tile_begins[side];
    if (tile_begin + wave >= tile_end) {
        if (Xnext != nullptr) request_first_tile<IO, D>(p, Xnext, xfirst, g, next_side, tile_begins[next_side], lane, wave);
        return;
    }
    Frag<IO, D> xs[AHEAD];
    xs[0] = xfirst;
#pragma unroll
    for (int a = 1; a < AHEAD; ++a) {
        const int tile = tile_begin + wave + a * WAVES;
        if (tile < tile_end) load_tokens<D>(xs[a], X + ((size_t)g * stride + min(tile * kTileTokens + io, n - 1)) * D, kg);
    }
#pragma unroll
    for (int slot = 0; slot < NT; ++slot) {
        const int tile = tile_begin + wave + slot * WAVES;
        if (tile < tile_end) {
            int skew = 0;
            asm volatile("" : "+v"(skew));
            f32x16 acc[RB];
            load_pivot_vector<RB>(acc, glds + skew, kg);
            if constexpr (similarity_by_pieces<IO, D, RB, WAVES>()) similarity_pieces<D, RB>(acc, zlds, xs[slot % AHEAD], lane, skew);
            else similarity<D, RB>(acc, zf, xs[slot % AHEAD]);
            if (slot + AHEAD < NT) {
                const int tnext = tile + AHEAD * WAVES;
                if (tnext < tile_end)
                    load_tokens<D>(xs[slot % AHEAD], X + ((size_t)g * stride + min(tnext * kTileTokens + io, n - 1)) * D, kg);
            }
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
            const float mc = pair_max(fmaxf(fmaxf(m0, m1), fmaxf(m2, m3))) * c1;
#pragma unroll
            for (int mb = 0; mb < RB; ++mb)
#pragma unroll
                for (int j = 0; j < 16; ++j) acc[mb][j] = exp2_fast(fmaf(acc[mb][j], c1, -mc));
            if constexpr (TO_LDS) {
                uint32_t packed[NW];
                res_pack<IO, RB>(packed, acc);
                res_to_lds<NW>(kres_wave + slot * (NW / 4) * 64, packed, lane);
            } else {
                res_pack<IO, RB>(kq[slot], acc);
            }
        }
        __builtin_amdgcn_sched_barrier(0);
    }
    if (Xnext != nullptr) request_first_tile<IO, D>(p, Xnext, xfirst, g, next_side, tile_begins[next_side], lane, wave);
}

// The kept matrix as operand of the matrix cores (bf16 I/O: two bf16 entries per register).  A lane's
// 8 RB words of a tile are, four at a time, its 8 numbers of one MFMA step over 16 pivots: step s covers
// the lane's accumulator registers 8 (s & 1) .. + 7 of pivot block s >> 1.  The row sums
// s_i = sum_t Kt_it v_t are then one small product per step with v as the other operand: rows of that
// operand alternate between the leading bf16 part of v (even rows) and the rest (odd rows), so that the
// first two result registers of every lane hold the two parts of its token's sum, over all pivots and to
// fp32 accuracy.  `vhl` points at [2][64] bf16: leading parts, then the rests.
template <int RB>
__device__ __forceinline__ void kept_v_fragments(bf16x8 (&vf)[2 * RB], const uint16_t* vhl, bool unit_v, int lane)
{
    const int kg = lane >> 5;
    const uint16_t* src = vhl + (lane & 1) * 64 + 4 * kg;
#pragma unroll
    for (int s = 0; s < 2 * RB; ++s) {
        const u32x2 a = *reinterpret_cast<const u32x2*>(src + 16 * s);
        const u32x2 b = *reinterpret_cast<const u32x2*>(src + 16 * s + 8);
        u32x4 t;
        t[0] = a[0]; t[1] = a[1]; t[2] = b[0]; t[3] = b[1];
        if (unit_v) {   // right after a fill: v = 1 (padding pivots hold zeros in the kept matrix)
            const uint32_t one = (lane & 1) ? 0u : 0x3f803f80u;
            t[0] = one; t[1] = one; t[2] = one; t[3] = one;
        }
        vf[s] = __builtin_bit_cast(bf16x8, t);
    }
}
template <int RB>
__device__ __forceinline__ f32x16 kept_row_sums(const bf16x8 (&vf)[2 * RB], const uint32_t (&w)[8 * RB])
{
    f32x16 d;
#pragma unroll
    for (int j = 0; j < 16; ++j) d[j] = 0.f;
#pragma unroll
    for (int s = 0; s < 2 * RB; ++s) {
        u32x4 t;
#pragma unroll
        for (int e = 0; e < 4; ++e) t[e] = w[4 * s + e];
        d = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[s], __builtin_bit_cast(bf16x8, t), d, 0, 0, 0);
    }
    return d;
}
// cs_t += Kt_it w for the lane's 16 RB pivots, straight from the packed words: a two-term bf16 dot
// product whose other operand is (w, 0) or (0, w).  w enters as bf16: its rounding (2^-9, zero mean,
// independent from token to token) averages out over the tokens of a column sum; the weights of the
// output rows and of the contraction with V are formed in fp32 elsewhere.  (These dot products were
// measured to share a pipe with the matrix instructions -- 32 of them and the four row-sum products of a
// tile take 340 cycles one after the other -- but unpacking and multiply-adds on the vector unit, for all
// or for half of the registers, measured slower in the kernel: 1.55-1.7 us per pass against 1.45-1.6.)
template <int RB>
__device__ __forceinline__ void kept_column_sums(f32x16 (&cs)[RB], const uint32_t (&w)[8 * RB], float weight)
{
    const uint32_t wb = (uint32_t)bf16_bits_of(weight);
    const bf16x2 w_even = __builtin_bit_cast(bf16x2, wb), w_odd = __builtin_bit_cast(bf16x2, wb << 16);
#pragma unroll
    for (int mb = 0; mb < RB; ++mb)
#pragma unroll
        for (int q = 0; q < 8; ++q) {
            const bf16x2 pr = __builtin_bit_cast(bf16x2, w[8 * mb + q]);
            cs[mb][2 * q] = __builtin_amdgcn_fdot2_f32_bf16(pr, w_even, cs[mb][2 * q], false);
            cs[mb][2 * q + 1] = __builtin_amdgcn_fdot2_f32_bf16(pr, w_odd, cs[mb][2 * q + 1], false);
        }
}

// A pass over the kept kernel matrix: no global memory, no exponential.  cs receives sum_i Kt_it / s_i
// per pivot; the caller multiplies the reduced sums by v_t.  fp32 I/O: vector arithmetic on the fp32
// entries.  bf16 I/O: the row sums on the matrix cores, straight from the packed words, and under way
// for the next tile while the vector unit forms the column sums of the current one.
// MASS: the tokens carry masses; nm[slot] = n times the mass of this lane's token of the wavefront's tile `slot`
// (kept in registers: fetched per pass, with one wavefront per SIMD, every tile would wait for memory -- measured
// 313 us against 191 on the streaming kernel at the headline shape); it multiplies what the token adds to the column sums.
template <typename IO, int RB, int WAVES, int NT, bool FROM_LDS, bool MASS>
__device__ __forceinline__ void cheap_pass(
    const FusedParams& p, int side, int tile_begin, int tile_end, int lane, int wave, const float* vlds,
    const uint16_t* vhl, bool unit_v,
    f32x16 (&cs)[RB], const uint32_t (&kq)[NT][(ResWords<IO, RB>::value)], const u32x4* kres_wave,
    const float (&nm)[MASS ? NT : 1])
{
    constexpr int NW = ResWords<IO, RB>::value;
    const int i = lane & 31, kg = lane >> 5;
    const int n = p.n_side[side];
    if constexpr (res_packed<IO>::value) {
        bf16x8 vf[2 * RB];
        kept_v_fragments<RB>(vf, vhl, unit_v, lane);
        const int mine = tile_end - tile_begin - wave;                 // tiles of this wavefront: ceil(mine / WAVES), at most NT
        if (mine <= 0) return;
        // (the row sums of slot + 1 are issued before the vector unit starts on slot: two result blocks in turn)
        auto words_of = [&](uint32_t (&w)[NW], int slot) __attribute__((always_inline)) {
            if constexpr (FROM_LDS) res_from_lds<NW>(w, kres_wave + slot * (NW / 4) * 64, lane);
            else {
#pragma unroll
                for (int q = 0; q < NW; ++q) w[q] = kq[slot][q];
            }
        };
        if (mine > (NT - 1) * WAVES && tile_end * kTileTokens <= n) {
            // every slot in use and no token past the end: no test inside
            uint32_t w[2][NW];
            f32x16 d[2];
            words_of(w[0], 0);
            d[0] = kept_row_sums<RB>(vf, w[0]);
#pragma unroll
            for (int slot = 0; slot < NT; ++slot) {
                if (slot + 1 < NT) {
                    words_of(w[(slot + 1) & 1], slot + 1);
                    d[(slot + 1) & 1] = kept_row_sums<RB>(vf, w[(slot + 1) & 1]);
                }
                const float weight = rcp_fast(d[slot & 1][0] + d[slot & 1][1]);
                kept_column_sums<RB>(cs, w[slot & 1], MASS ? weight * nm[MASS ? slot : 0] : weight);
            }
            return;
        }
#pragma unroll
        for (int slot = 0; slot < NT; ++slot) {
            const int tile = tile_begin + wave + slot * WAVES;
            if (tile < tile_end) {
                uint32_t w[NW];
                words_of(w, slot);
                const f32x16 d = kept_row_sums<RB>(vf, w);
                const int tok = tile * kTileTokens + i;
                kept_column_sums<RB>(cs, w, tok < n ? rcp_fast(d[0] + d[1]) * (MASS ? nm[MASS ? slot : 0] : 1.f) : 0.f);
            }
        }
        return;
    } else {
    f32x16 v[RB];
    load_pivot_vector<RB>(v, vlds, kg);
    if (unit_v) {      // right after a fill: the potentials are inside the kept matrix (padding pivots hold zeros there)
#pragma unroll
        for (int mb = 0; mb < RB; ++mb)
#pragma unroll
            for (int j = 0; j < 16; ++j) v[mb][j] = 1.f;
    }
    constexpr int kUnrollSlots = (FROM_LDS && !MASS) ? 1 : NT;   // unrolled only where the slot picks registers
#pragma unroll kUnrollSlots
    for (int slot = 0; slot < NT; ++slot) {
        const int tile = tile_begin + wave + slot * WAVES;
        if (tile < tile_end) {
            f32x16 k[RB];
            if constexpr (FROM_LDS) {
                uint32_t packed[NW];
                res_from_lds<NW>(packed, kres_wave + slot * (NW / 4) * 64, lane);
                res_unpack<IO, RB>(k, packed);
            } else {
                res_unpack<IO, RB>(k, kq[slot]);
            }
            float s0 = 0.f, s1 = 0.f, s2 = 0.f, s3 = 0.f;
#pragma unroll
            for (int mb = 0; mb < RB; ++mb)
#pragma unroll
                for (int j = 0; j < 16; j += 4) {
                    s0 = fmaf(k[mb][j], v[mb][j], s0);
                    s1 = fmaf(k[mb][j + 1], v[mb][j + 1], s1);
                    s2 = fmaf(k[mb][j + 2], v[mb][j + 2], s2);
                    s3 = fmaf(k[mb][j + 3], v[mb][j + 3], s3);
                }
            const float s = pair_sum((s0 + s1) + (s2 + s3));
            const int tok = tile * kTileTokens + i;
            const float w = tok < n ? rcp_fast(s) * (MASS ? nm[MASS ? slot : 0] : 1.f) : 0.f;
#pragma unroll
            for (int mb = 0; mb < RB; ++mb)
#pragma unroll
                for (int j = 0; j < 16; ++j) cs[mb][j] = fmaf(k[mb][j], w, cs[mb][j]);
        }
    }
    }
}

// The last key pass over the kept kernel matrix: the work of cheap_pass plus U = sum_j (Kt_jt / s_j) V_j
// by MFMA (the factor v_t is left out here as well; the caller applies it to the rows of U).  The
// coupling tile is transposed through LDS like in run_pass; the transposition area is the beginning of
// this wavefront's own block of kept data, which is why the words of the next slot are fetched before
// the current slot's transposed tile is written (block layout: see the kernel).  The value rows of AHEAD
// tiles are kept in flight: this is the only pass of these variants that reads memory it has not asked
// for long before, and with one wavefront per SIMD nobody else runs while it waits.
template <typename IO, int D, int RB, int WAVES, int NT, int AHEAD, bool MASS>
__device__ __forceinline__ void accum_from_kept(
    const FusedParams& p, const IO* __restrict__ V, int g, int tile_begin, int tile_end, int lane, int wave,
    const float* vlds, const uint16_t* vhl, bool unit_v, f32x16 (&cs)[RB], f32x16 (&U)[RB][D / 32], char* block,
    const float (&nm)[MASS ? NT : 1])
{
    constexpr int NW = ResWords<IO, RB>::value;
    constexpr int NB = D / 32;
    constexpr bool kSplit = io_is_f32<IO>::value;
    constexpr bool kAhead = AHEAD > 1;       // value rows of several tiles in flight, row sums on the matrix cores
    static_assert(!kAhead || res_packed<IO>::value, "the deep variant is written for bf16 I/O");
    // (an opaque copy of the lane index for the addresses of the value rows: formed from the plain one, the
    // addresses of all slots are hoisted out of the iteration loop and spilled)
    int lane_o = lane;
    asm volatile("" : "+v"(lane_o));
    const int io = lane_o & 31, kgo = lane_o >> 5;
    const int i = lane & 31, kg = lane >> 5;
    const int n = p.n_side[0];
    const int stride = p.stride_side[0];
    const u32x4* kres_wave = reinterpret_cast<const u32x4*>(block);
    uint16_t* tr_hi = reinterpret_cast<uint16_t*>(block);
    uint16_t* tr_lo = tr_hi + 32 * RB * kTrStride;
    if (tile_begin + wave >= tile_end) return;
    bf16x8 vf[kAhead ? 2 * RB : 1];
    if constexpr (kAhead) kept_v_fragments<RB>(vf, vhl, unit_v, lane);
    uint32_t raw[kAhead ? AHEAD : 1][16];
    const bool inside = tile_end * kTileTokens <= n;   // no token of this workgroup's tiles is past the end
    auto request_values = [&](int buf, int tile) __attribute__((always_inline)) {
        if constexpr (kAhead) {
            const uint16_t* Vu = reinterpret_cast<const uint16_t*>(V);
            if (inside) {
                request_value_rows_inside<D>(raw[buf], Vu + ((size_t)g * stride + tile * kTileTokens + 8 * kgo) * D + (D / 32) * io);
            } else {
                const int t0 = tile * kTileTokens + 8 * kgo;
                request_value_rows<D>(raw[buf], Vu, io, [&](int s, int e) -> size_t {
                    return (size_t)g * stride + min(t0 + 16 * s + e, n - 1);
                });
            }
        }
    };
    if constexpr (kAhead) {
#pragma unroll
        for (int a = 0; a < AHEAD; ++a) {
            const int tile = tile_begin + wave + a * WAVES;
            if (a < NT && tile < tile_end) request_values(a, tile);
        }
    }
    uint32_t cur[NW], nxt[NW];
    res_from_lds<NW>(cur, kres_wave, lane);
#pragma unroll
    for (int q = 0; q < NW; ++q) nxt[q] = 0u;
    constexpr int kUnrollSlots = (kAhead || MASS) ? NT : 1;   // unrolled only where the slot picks registers (value rows, masses)
#pragma unroll kUnrollSlots
    for (int slot = 0; slot < NT; ++slot) {
        const int tile = tile_begin + wave + slot * WAVES;
        if (tile < tile_end) {
            if (slot + 1 < NT && tile + WAVES < tile_end) res_from_lds<NW>(nxt, kres_wave + (slot + 1) * (NW / 4) * 64, lane);
            bf16x8 vh[2][NB], vl[2][NB];
            if constexpr (!kAhead) {
                // (requested now, used at the end of the tile)
#pragma unroll
                for (int s = 0; s < 2; ++s) {
                    const int t0 = tile * kTileTokens + 16 * s + 8 * kg;
                    const int left = max(1, min(8, n - t0));
                    load_values<D>(vh[s], vl[s], V, (size_t)g * stride + min(t0, n - 1), left, i);
                }
            }
            f32x16 k[RB];
            res_unpack<IO, RB>(k, cur);
            float s;
            if constexpr (kAhead) {
                const f32x16 d = kept_row_sums<RB>(vf, cur);
                s = d[0] + d[1];
            } else {
                float s0 = 0.f, s1 = 0.f, s2 = 0.f, s3 = 0.f;
                if (unit_v) {
#pragma unroll
                    for (int mb = 0; mb < RB; ++mb)
#pragma unroll
                        for (int j = 0; j < 16; j += 4) { s0 += k[mb][j]; s1 += k[mb][j + 1]; s2 += k[mb][j + 2]; s3 += k[mb][j + 3]; }
                } else {
#pragma unroll
                    for (int mb = 0; mb < RB; ++mb)
#pragma unroll
                        for (int q = 0; q < 4; ++q) {
                            const f32x4 v = *reinterpret_cast<const f32x4*>(vlds + 32 * mb + 8 * q + 4 * kg);
                            s0 = fmaf(k[mb][4 * q], v[0], s0);
                            s1 = fmaf(k[mb][4 * q + 1], v[1], s1);
                            s2 = fmaf(k[mb][4 * q + 2], v[2], s2);
                            s3 = fmaf(k[mb][4 * q + 3], v[3], s3);
                        }
                }
                s = pair_sum((s0 + s1) + (s2 + s3));
            }
            const int tok = tile * kTileTokens + i;
            float w = tok < n ? rcp_fast(s) : 0.f;
            if constexpr (MASS) w *= nm[MASS ? slot : 0];   // the keys' masses weight U as well
            // (the words of this slot and of the next are in registers: their bytes may be overwritten now)
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
#pragma unroll
            for (int mb = 0; mb < RB; ++mb)
#pragma unroll
                for (int j = 0; j < 16; ++j) {
                    const float x = k[mb][j] * w;
                    cs[mb][j] += x;
                    const __bf16 h = (__bf16)x;
                    const int pv = pivot_of(mb, j, kg);
                    tr_hi[pv * kTrStride + i] = __builtin_bit_cast(uint16_t, h);
                    if (kSplit) tr_lo[pv * kTrStride + i] = __builtin_bit_cast(uint16_t, (__bf16)(x - (float)h));
                }
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
            if constexpr (kAhead) value_fragments<D>(vh, raw[slot % AHEAD]);   // (the first use of what was fetched AHEAD tiles ago)
#pragma unroll
            for (int s2i = 0; s2i < 2; ++s2i) {
#pragma unroll
                for (int mb = 0; mb < RB; ++mb) {
                    const bf16x8 ah = *reinterpret_cast<const bf16x8*>(tr_hi + (32 * mb + i) * kTrStride + 16 * s2i + 8 * kg);
#pragma unroll
                    for (int nb = 0; nb < NB; ++nb)
                        U[mb][nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ah, vh[s2i][nb], U[mb][nb], 0, 0, 0);
                    if (kSplit) {
                        const bf16x8 al = *reinterpret_cast<const bf16x8*>(tr_lo + (32 * mb + i) * kTrStride + 16 * s2i + 8 * kg);
#pragma unroll
                        for (int nb = 0; nb < NB; ++nb) {
                            U[mb][nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(al, vh[s2i][nb], U[mb][nb], 0, 0, 0);
                            U[mb][nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ah, vl[s2i][nb], U[mb][nb], 0, 0, 0);
                        }
                    }
                }
            }
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            if constexpr (kAhead) {
                if (slot + AHEAD < NT && tile + AHEAD * WAVES < tile_end) request_values(slot % AHEAD, tile + AHEAD * WAVES);
            }
#pragma unroll
            for (int q = 0; q < NW; ++q) cur[q] = nxt[q];
        }
        if constexpr (kAhead) __builtin_amdgcn_sched_barrier(0);
    }
}

// The expansion O = n Gamma1 Y' from the queries' kept kernel matrix: row weights Kt_it / s_i times
// Y''_t, which the caller has scaled by v_t as well (so the weights need no factor per pivot).
template <typename IO, int D, int RB, int WAVES, int NT>
__device__ __forceinline__ void expand_from_kept(
    const FusedParams& p, int g, int tile_begin, int tile_end, int lane, int wave, const float* vlds, bool unit_v,
    const uint32_t (&kq)[NT][(ResWords<IO, RB>::value)], const bf16x8* yf_hi, const bf16x8* yf_lo, IO* __restrict__ out)
{
    constexpr int NB = D / 32;
    constexpr bool kSplit = io_is_f32<IO>::value;
    const int i = lane & 31, kg = lane >> 5;
    const int n = p.n_side[1];
    const int stride = p.stride_side[1];
#pragma unroll
    for (int slot = 0; slot < NT; ++slot) {
        const int tile = tile_begin + wave + slot * WAVES;
        if (tile < tile_end) {
            f32x16 k[RB];
            res_unpack<IO, RB>(k, kq[slot]);
            float s0 = 0.f, s1 = 0.f, s2 = 0.f, s3 = 0.f;
            if (unit_v) {
#pragma unroll
                for (int mb = 0; mb < RB; ++mb)
#pragma unroll
                    for (int j = 0; j < 16; j += 4) { s0 += k[mb][j]; s1 += k[mb][j + 1]; s2 += k[mb][j + 2]; s3 += k[mb][j + 3]; }
            } else {
#pragma unroll
                for (int mb = 0; mb < RB; ++mb)
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        const f32x4 v = *reinterpret_cast<const f32x4*>(vlds + 32 * mb + 8 * q + 4 * kg);
                        s0 = fmaf(k[mb][4 * q], v[0], s0);
                        s1 = fmaf(k[mb][4 * q + 1], v[1], s1);
                        s2 = fmaf(k[mb][4 * q + 2], v[2], s2);
                        s3 = fmaf(k[mb][4 * q + 3], v[3], s3);
                    }
            }
            const float s = pair_sum((s0 + s1) + (s2 + s3));
            const float w = rcp_fast(s);
            f32x16 oacc[NB];
#pragma unroll
            for (int nb = 0; nb < NB; ++nb)
#pragma unroll
                for (int j = 0; j < 16; ++j) oacc[nb][j] = 0.f;
#pragma unroll
            for (int st = 0; st < 2 * RB; ++st) {
                f32x8 wv;
#pragma unroll
                for (int e = 0; e < 8; ++e) wv[e] = k[st >> 1][8 * (st & 1) + e] * w;
                bf16x8 ah, al;
                if (kSplit) split_bf16(wv, ah, al);
                else ah = __builtin_convertvector(wv, bf16x8);
#pragma unroll
                for (int nb = 0; nb < NB; ++nb) {
                    const bf16x8 yh = yf_hi[(st * NB + nb) * 64 + lane];
                    oacc[nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ah, yh, oacc[nb], 0, 0, 0);
                    if (kSplit) {
                        const bf16x8 yl = yf_lo[(st * NB + nb) * 64 + lane];
                        oacc[nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(al, yh, oacc[nb], 0, 0, 0);
                        oacc[nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ah, yl, oacc[nb], 0, 0, 0);
                    }
                }
            }
            const int row0 = tile * kTileTokens + 4 * kg;
            IO* const lane_base = out + ((size_t)g * stride + row0) * D;
            if ((tile + 1) * kTileTokens <= n) {
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
    }
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
template <typename IO, int D, int RB, int WAVES, int NT, bool MASS = false>
__global__ void __launch_bounds__(WAVES * 64, 2) lot_fused_kernel(FusedParams p)
{
    constexpr int NB = D / 32;
    constexpr int kThreads = WAVES * 64;
    constexpr int NW = ResWords<IO, RB>::value;
    constexpr bool kKept = NT > 0;
    constexpr bool kSplitIO = io_is_f32<IO>::value;
    // Wavefronts of a workgroup that post its column sums to the problem's accumulators.  With four
    // wavefronts, each of the three that reduce posts its own share.  With eight, seven posts per
    // workgroup were measured to cost more than they save (the acknowledgements of so many atomics on the
    // same words take microseconds, and every reload of a spilled register in the next pass waits for
    // them): the seven leave their shares in LDS and one of them posts the sum.
    constexpr int kPosters = WAVES == 4 ? WAVES - 1 : 1;
    // NT == 0: s_u holds the workgroup's sum of U, s_big the transposition areas of the two contraction
    // passes (every wavefront its own, hi and lo), later the fragments of Y''.
    // NT > 0: s_big is one block per wavefront.  A block holds the wavefront's share of the keys' kernel
    // matrix, slot after slot; the last key pass uses the beginning of the same block as its transposition
    // area (at most two slots long: it fetches one slot ahead), and once every wavefront is through
    // that pass the whole area is free: it then takes s_u (at the front), the buffers of the U reduction
    // and the fragments of Y'' (behind s_u).
    constexpr int kTrBytes = WAVES * 2 * 64 * kTrStride * 2;
    constexpr int kSlotBytes = NW * 64 * 4;
    constexpr int kTrWave = (kSplitIO ? 2 : 1) * 32 * RB * kTrStride * 2;
    constexpr int kBlockBytes = NT * kSlotBytes > kTrWave ? NT * kSlotBytes : kTrWave;
    constexpr int kUBytes = 64 * D * 4;
    constexpr int kYfBytes = 2 * (2 * RB * NB * 64) * 16;
    // (room for several buffers in the U reduction, up to 64 KB of them: few rounds)
    constexpr int kMoreBufs = (WAVES - 1) * kUBytes < 65536 ? (WAVES - 1) * kUBytes : 65536;
    constexpr int kAfterBytes = kUBytes + (kYfBytes > kMoreBufs ? kYfBytes : kMoreBufs);
    constexpr int kKeptBytes = WAVES * kBlockBytes > kAfterBytes ? WAVES * kBlockBytes : kAfterBytes;
    constexpr int kBigBytes = kKept ? kKeptBytes : kTrBytes;
    static_assert(!kKept || NT == 1 || kTrWave <= 2 * kSlotBytes, "the transposed tile must fit the two slots already fetched");
    __shared__ float s_wave_part[2][WAVES][64];   // per side: the reader of one pass never meets the writers of the next
    __shared__ __attribute__((aligned(16))) float s_hand[16 * RB * 64];   // the first wavefront's column sums, on their way to the others
    __shared__ float s_g[2][64];       // pivot potentials per side (0 = keys, 1 = queries)
    __shared__ float s_rho[2][64];     // beta_t / colsum_t after the last iteration
    __shared__ float s_csinv[64];      // 1 / colsum_t of the key side after the last iteration
    __shared__ float s_beta[64];
    __shared__ __attribute__((aligned(16))) float s_u_own[kKept ? 4 : 64 * D];
    __shared__ __attribute__((aligned(16))) char s_big[kBigBytes];
    float* const s_u = kKept ? reinterpret_cast<float*>(s_big) : s_u_own;
    uint16_t* const s_tr = reinterpret_cast<uint16_t*>(s_big);
    // NT > 0 with bf16 I/O: the pivots as MFMA operand fragments (fp32 I/O keeps their bf16 pieces in s_zf)
    __shared__ __attribute__((aligned(16))) char s_zst[kKept && !similarity_by_pieces<IO, D, RB, WAVES>() ? RB * (D / 16) * 64 * 16 : 16];
    __shared__ float s_gref[2][64];    // NT > 0: the potentials folded into the kept kernel matrix, per side
    __shared__ float s_v[2][64];       // NT > 0: exp((g - gref)/eps - shift) per side
    __shared__ __attribute__((aligned(16))) uint16_t s_vhl[2][2][64];   // ... as bf16: leading part, rest (operand of the row-sum products)
    __shared__ int s_fill[2];          // NT > 0: the next pass of this side must recompute the kernel matrix
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
    uint16_t* tr_hi = s_tr + (wave * 2 + 0) * 64 * kTrStride;      // (NT == 0 only)
    uint16_t* tr_lo = s_tr + (wave * 2 + 1) * 64 * kTrStride;
    bf16x8* yf_hi = reinterpret_cast<bf16x8*>(s_big + (kKept ? kUBytes : 0));
    bf16x8* yf_lo = yf_hi + 2 * RB * NB * 64;
    const bool attention = p.mode == MODE_ATTENTION;

    // Block ids go round the 8 XCDs of the device.  When the grid is one item per workgroup and a multiple
    // of 8, the items are dealt so that consecutive ones -- the workgroups of one problem, which exchange
    // sums all the time -- sit on one XCD (measured: a round of the counted exchange between 16 workgroups
    // takes 0.68 us there against 0.94 us when they are spread over the dies).  Any other mapping is as
    // correct; this one is only nearer.
    const bool dealt = (int)gridDim.x == p.num_items && (gridDim.x & 7u) == 0u;
    const int first_item = dealt ? (int)((blockIdx.x & 7u) * (gridDim.x >> 3) + (blockIdx.x >> 3)) : (int)blockIdx.x;
    for (int item = first_item; item < p.num_items; item += gridDim.x) {
        LOT_STAMP(0);
#ifdef LOT_TRACE
        unsigned long long clk0 = 0;
        if (threadIdx.x == 0 && p.trace) clk0 = clock64();
#endif
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
        } else if constexpr (kKept) {
            if (wave == 0) stash_pivots<D, RB>(s_zst, zf, lane);
        }
        if (tid < 128) s_g[tid >> 6][tid & 63] = (tid & 63) < r ? 0.f : kNegBig;
        if constexpr (NT > 0) {
            if (tid < 128) {
                s_gref[tid >> 6][tid & 63] = 0.f;
                s_v[tid >> 6][tid & 63] = (tid & 63) < r ? 1.f : 0.f;
                s_vhl[tid >> 6][0][tid & 63] = (tid & 63) < r ? (uint16_t)0x3f80u : (uint16_t)0u;
                s_vhl[tid >> 6][1][tid & 63] = 0;
            }
            if (tid < 2) s_fill[tid] = 0;
        }
        if (tid < 64) s_beta[tid] = tid < r ? beta_read : 1.f;
        if (tid < 256) (&s_prev[0][0][0])[tid] = 0ull;   // the accumulators start at zero in every launch
        if (blockIdx.x == 0 && tid == 0 && item == first_item)
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
            // (everything this needs from LDS is asked for first: the answers arrive while the poll is awaited)
            const unsigned long long prev = p.cluster > 1 ? s_prev[side][it & 1][ln] : 0ull;
            const float b = s_beta[ln];
            const float g_old = s_g[side][ln];
            float gref = 0.f;
            if constexpr (NT > 0) gref = s_gref[side][ln];
            float tot = 0.f;
            bool ok = true;
            if (p.cluster > 1) {
                // every pivot's word carries its own arrival count: complete when all 64 agree
                const unsigned long long* src = p.colacc + (((size_t)2 * g + side) * 2 + (it & 1)) * 64 + ln;
                unsigned long long word = early;   // a poll that was started ahead; validated here
                const unsigned arrivals = (unsigned)p.cluster * (unsigned)kPosters;
                ok = __all(((unsigned)((word >> kCountShift) - (prev >> kCountShift)) & kCountMask) == arrivals);
#ifdef LOT_TRACE
                valid_a += ok ? 1 : 0;
#endif
                for (uint32_t k = 0; !ok && k < p.spin_limit; ++k) {
#ifdef LOT_TRACE
                    ++repolls;
#endif
                    word = __hip_atomic_load(src, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    if (__all(((unsigned)((word >> kCountShift) - (prev >> kCountShift)) & kCountMask) == arrivals)) { ok = true; break; }
                    if ((k & 63u) == 63u && gave_up(p.status, p.nonce)) break;
                    __builtin_amdgcn_s_sleep(1);
                }
                s_prev[side][it & 1][ln] = word;
                const unsigned long long mask = (1ull << kCountShift) - 1ull;
                tot = (float)(long long)((word & mask) - (prev & mask)) * p.fx_unscale;
                if (!ok && ln == 0) give_up(p.status, p.nonce);
            } else {
                // a single workgroup: the totals its wavefronts left in LDS (fixed order of the additions)
                tot = s_wave_part[side][1][ln];
#pragma unroll
                for (int wv = 2; wv < WAVES; ++wv) tot += s_wave_part[side][wv][ln];
            }
            float g_new = g_old;
            if (ln < rr) {
                // (sums exchanged in fixed point: one below the resolution reads as half a unit)
                const float c = fmaxf(tot, p.cluster > 1 ? 0.5f * p.fx_unscale : 1.0e-37f);
                // (hardware reciprocal and base-2 logarithm, each good to one unit in the last place: this
                // runs on one wavefront while the others wait for the potentials)
                const float cinv = rcp_fast(c);
                if (!final) {
                    g_new = g_old + (p.eps * kLn2) * __builtin_amdgcn_logf((float)opaque_scalar(p.n_side[side]) * b * cinv);
                    s_g[side][ln] = g_new;
                } else {
                    // the last pass's potentials stay: the epilogue rebuilds its coupling from them
                    s_rho[side][ln] = b * cinv;
                    if (side == 0) s_csinv[ln] = cinv;
                }
            } else if (final) {
                s_rho[side][ln] = 0.f;
                if (side == 0) s_csinv[ln] = 0.f;
            }
            if constexpr (NT > 0) {
                if (!final) {
                    // how far the potentials have moved from those folded into the kept kernel matrix
                    // Any common shift will do for v as long as nothing leaves the fp32 range: that of
                    // pivot 0.  As long as every pivot stays within kDriftLimit / 2 binary orders of it, the
                    // spread is within kDriftLimit; otherwise (or when something is not finite) the next pass
                    // of this side recomputes the kernel matrix.
                    const bool lv = ln < rr;
                    const float d = (g_new - gref) * c1;
                    const float d0 = __builtin_bit_cast(float, __builtin_amdgcn_readfirstlane(__builtin_bit_cast(int, d)));
                    const float rel = d - d0;
                    const float vv = lv ? exp2_fast(rel) : 0.f;
                    s_v[side][ln] = vv;
                    if constexpr (res_packed<IO>::value) {
                        const __bf16 vh = (__bf16)vv;
                        s_vhl[side][0][ln] = __builtin_bit_cast(uint16_t, vh);
                        s_vhl[side][1][ln] = bf16_bits_of(vv - (float)vh);
                    }
                    const bool any_far = __any(lv && !(fabsf(rel) <= p.drift_half));   // (all 64 lanes take part)
                    if (ln == 0) s_fill[side] = any_far ? 1 : 0;
                }
            }
            return ok;
        };

        // ---- after a pass: post this workgroup's share (column sums; U on the last key pass) and,
        //      in the same breath, collect the other side's previous pass, which was posted one
        //      whole pass ago.  One workgroup barrier in all (more when U is reduced).
        // (always inlined: where with_u is the constant false, as in the copies inside the iteration loop of
        // the kept-matrix variants, the 64 registers of U are then not kept alive)
        auto exchange = [&](int side, int it, bool with_u, int cside, int cit, bool cfinal, bool cheap) __attribute__((always_inline)) -> bool {
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
                // start the poll now; it completes during the hand-over.  (Started inside the pass -- into a
                // register or straight into LDS -- it would be there in time, but every reload of a spilled
                // register in the pass then waits for it as well: measured, the sweeps take 2.3-2.6 us instead
                // of 1.5.  Sent off before the pass, into LDS, it mostly finds the sums incomplete, and the
                // second poll then costs a whole round trip: 0.9 us per collect instead of 0.7.)
                early_word = ldc_u64(coherent_view(p.colacc),
                                     (uint32_t)(((((size_t)2 * g + cside) * 2 + (cit & 1)) * 64 + lane) * 8));
                // after the very last pass the query side is collected as well
                if (side == 1 && it == p.iters)
                    early_word2 = ldc_u64(coherent_view(p.colacc),
                                          (uint32_t)(((((size_t)2 * g + 1) * 2 + (it & 1)) * 64 + lane) * 8));
            }
            // The first wavefront hands its column sums to the others through LDS and turns to the other
            // side's sums at once (they do not depend on this pass at all); the others add their shares of
            // what it left, reduce over the tokens (one pivot per lane after the transposing reduction) and
            // post: one fire-and-forget atomic per pivot and wavefront, the sum in fixed point (integer
            // addition: the total does not depend on arrival order) plus one count.  Two workgroup barriers:
            // the hand-over, and the publication of the updated potentials.
            constexpr int kUnits = 4 * RB;                         // 16-byte units of a lane's accumulators
            f32x4* const hand = reinterpret_cast<f32x4*>(s_hand);
            if (wave == 0) {
#pragma unroll
                for (int u = 0; u < kUnits; ++u) {
                    f32x4 t;
#pragma unroll
                    for (int e = 0; e < 4; ++e) t[e] = cs[u >> 2][4 * (u & 3) + e];
                    hand[u * 64 + lane] = t;
                }
            }
            lds_barrier();
            LOT_STAMP(10 + 6 * ((it - 1) * 2 + side));   // handed over
            if (wave == 0) {
                bool ok = true;
                if (cit >= 1) ok = collect_w0(cside, cit, cfinal, early_word);
                if (fresh_lane() == 0) s_okx[side] = ok;
                LOT_STAMP(11 + 6 * ((it - 1) * 2 + side));   // collected
            } else {
                const int u0 = (wave - 1) * kUnits / (WAVES - 1), u1 = wave * kUnits / (WAVES - 1);
#pragma unroll
                for (int u = 0; u < kUnits; ++u)
                {
                        const f32x4 t = hand[u * 64 + lane];
                        const float m = (u >= u0 && u < u1) ? 1.f : 0.f;
#pragma unroll
                        for (int e = 0; e < 4; ++e) cs[u >> 2][4 * (u & 3) + e] = fmaf(t[e], m, cs[u >> 2][4 * (u & 3) + e]);
                    }
                float c[16 * RB];
#pragma unroll
                for (int mb = 0; mb < RB; ++mb)
#pragma unroll
                    for (int j = 0; j < 16; ++j) c[16 * mb + j] = cs[mb][j];
                float tot = reduce_scatter_tokens<16 * RB>(c, i);
                const int q = RB == 2 ? i : i >> 1;   // accumulator register this lane ended up with
                const int pv = 32 * (q >> 4) + 8 * ((q & 15) >> 2) + 4 * kg + (q & 3);
                if (pv >= opaque_scalar(r)) tot = 0.f;   // padding pivots
                if constexpr (NT > 0) {
                    if (cheap) tot *= s_v[side][pv];     // a pass over the kept kernel matrix leaves the factor v_t out
                }
                // (RB == 1: two lanes hold every total.  One of them posts it; the other posts a zero to the
                // word 32 further on, which belongs to no pivot: the collecting wavefront waits for all 64 counts)
                const bool second = RB == 1 && (i & 1) != 0;
                const int word_of = second ? 32 + pv : pv;
                if (second) tot = 0.f;
                if (p.cluster > 1 && kPosters > 1) {
                    const unsigned long long word = (1ull << kCountShift) + (unsigned long long)__float2ll_rn(tot * p.fx_scale);
                    __hip_atomic_fetch_add(p.colacc + (((size_t)2 * g + side) * 2 + (it & 1)) * 64 + word_of, word,
                                           __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                } else {
                    s_wave_part[side][wave][word_of] = tot;
                }
                LOT_STAMP(11 + 6 * ((it - 1) * 2 + side));   // (a posting wavefront: posted)
            }
            if (with_u) {
                // Workgroup total of U in s_u.  The wavefronts dump their accumulators into separate
                // buffers (s_u itself and the now idle transposition area), in rounds when there are
                // more wavefronts than buffers; then every thread sums its elements over the buffers.
                // The order of the additions is fixed.
                constexpr int kElems = 64 * D;
                constexpr int kExtra = (int)((kKept ? kBigBytes - kUBytes : kTrBytes) / (kElems * sizeof(float)));
                constexpr int kBufs = WAVES < 1 + kExtra ? WAVES : 1 + kExtra;
                float* const extra = reinterpret_cast<float*>(s_big + (kKept ? kUBytes : 0));
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
            LOT_STAMP(12 + 6 * ((it - 1) * 2 + side));   // potentials published
            if (kPosters == 1 && p.cluster > 1 && wave == 1) {
                // one post per workgroup: the second wavefront adds up what the others left (fixed order)
                const int ln = fresh_lane();
                float tot = s_wave_part[side][1][ln];
#pragma unroll
                for (int wv = 2; wv < WAVES; ++wv) tot += s_wave_part[side][wv][ln];
                const unsigned long long word = (1ull << kCountShift) + (unsigned long long)__float2ll_rn(tot * p.fx_scale);
                __hip_atomic_fetch_add(p.colacc + (((size_t)2 * g + side) * 2 + (it & 1)) * 64 + ln, word,
                                       __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
            if (with_u && p.cluster > 1) {
                float* up = p.u_part + ((size_t)g * p.cluster_cap + chunk) * 64 * D;
                for (int e = wave * 64 + fresh_lane(); e < 64 * D; e += kThreads) st_coherent(up + e, s_u[e]);
                publish_barrier();   // the stores above have been acknowledged
                if (tid == 0) __hip_atomic_fetch_add(p.arrive + g, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
            __builtin_amdgcn_s_setprio(0);
            return s_okx[side] != 0;
        };

        // ---- cluster-wide sum of U: once every workgroup of the cluster has posted its share, each sums
        //      one slice of them (raw, still unnormalised) and publishes it.  False if a wait gave up.
        float* yt = p.y_tile + (size_t)g * 64 * D;
        auto reduce_u_slice = [&]() __attribute__((always_inline)) -> bool {
            __builtin_amdgcn_s_setprio(3);
            if (tid == 0) {
                const bool ok = spin_until(p.arrive + g, (uint32_t)p.cluster, p.status, p.nonce, p.spin_limit);
                if (!ok) give_up(p.status, p.nonce);
                s_ok = ok;
            }
            lds_barrier();
            if (!s_ok) return false;
            const int per = (64 * D + p.cluster - 1) / p.cluster;
            const int e0 = chunk * per, e1 = min(64 * D, e0 + per);
            const float* up = p.u_part + (size_t)g * p.cluster_cap * 64 * D;
            const __amdgpu_buffer_rsrc_t upv = coherent_view(up);
            for (int e = e0 + wave * 64 + fresh_lane(); e < e1; e += kThreads) {
                float acc = 0.f;
                // (sixteen loads in flight at a time: every batch is one round trip to memory)
                for (int k0 = 0; k0 < p.cluster; k0 += 16) {
                    float v[16];
#pragma unroll
                    for (int j = 0; j < 16; ++j)
                        v[j] = ldc_f32(upv, (uint32_t)(((size_t)min(k0 + j, p.cluster - 1) * 64 * D + e) * 4));
#pragma unroll
                    for (int j = 0; j < 16; ++j) acc += (k0 + j < p.cluster) ? v[j] : 0.f;
                }
                st_coherent(yt + e, acc);
            }
            publish_barrier();   // the slice has been acknowledged
            if (tid == 0) __hip_atomic_fetch_add(p.yready + g, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            __builtin_amdgcn_s_setprio(0);
            return true;
        };

        bool unit_k = false, unit_q = false;   // NT > 0: the last pass of that side refilled the kernel matrix (v = 1)
        uint32_t kq[kKept ? NT : 1][NW];
        if constexpr (NT > 0) {
            // ---- the kernel matrix stays on chip: queries in registers, keys in LDS
#pragma unroll
            for (int sl = 0; sl < NT; ++sl)
#pragma unroll
                for (int q = 0; q < NW; ++q) kq[sl][q] = 0u;
            char* const block = s_big + (size_t)wave * kBlockBytes;
            u32x4* const kres_wave = reinterpret_cast<u32x4*>(block);
            // n times the mass of this lane's token of every tile of the wavefront, per side (a side without masses
            // of its own: 1; a token past the end takes the last one's, its weight is 0 anyway)
            float nmass[2][MASS ? NT : 1];
            if constexpr (MASS) {
#pragma unroll
                for (int sd = 0; sd < 2; ++sd) {
                    const float* const ms = p.mass_side[sd];
                    const int ns = p.n_side[sd];
#pragma unroll
                    for (int sl = 0; sl < NT; ++sl) {
                        const int tok = min((tile_begins[sd] + wave + sl * WAVES) * kTileTokens + i, ns - 1);
                        nmass[sd][sl] = ms != nullptr ? (float)ns * as_global(ms)[(size_t)g * ns + tok] : 1.f;
                    }
                }
            }
            const void* const zlds = similarity_by_pieces<IO, D, RB, WAVES>() ? (const void*)s_zf : (const void*)s_zst;
            bool have_first = true;     // xfirst holds the first key tile
            // One pass and its exchange.  The last key pass (with_u_c = true_type: it also contracts with V) is
            // a separate copy of this code, outside the iteration loop.
            for (int it = 1; it <= p.iters; ++it) {
                for (int side = 0; side < 2; ++side) {
#pragma unroll
                    for (int mb = 0; mb < RB; ++mb)
#pragma unroll
                        for (int j = 0; j < 16; ++j) cs[mb][j] = 0.f;
                    const bool fill = it == 1 || __builtin_amdgcn_readfirstlane(s_fill[side]) != 0;
                    LOT_STAMP(8 + 6 * ((it - 1) * 2 + side));   // pass starts
                    if (fill) {
                        if (!have_first) request_first_tile<IO, D>(p, Xs[side], xfirst, g, side, tile_begins[side], lane, wave);
                        // the only fill that is always followed by another one: the keys' first pass
                        const bool next_too = side == 0 && it == 1;
                        const IO* Xnext = next_too ? Xs[1] : nullptr;
                        if (wave == 0) s_gref[side][fresh_lane()] = s_g[side][fresh_lane()];
                        if constexpr (WAVES == 4 && NT >= 4) {
                            if (side == 0) fill_pass_ahead<IO, D, RB, WAVES, NT, true, 4>(p, Xs[0], Xnext, 1, xfirst, g, 0, tile_begins, tile_ends[0], lane, wave, c1, zlds, s_g[0], kq, kres_wave);
                            else fill_pass_ahead<IO, D, RB, WAVES, NT, false, 4>(p, Xs[1], Xnext, 1, xfirst, g, 1, tile_begins, tile_ends[1], lane, wave, c1, zlds, s_g[1], kq, kres_wave);
                        } else {
                            if (side == 0) fill_pass<IO, D, RB, WAVES, NT, true>(p, Xs[0], Xnext, 1, xfirst, g, 0, tile_begins, tile_ends[0], lane, wave, c1, zlds, s_g[0], kq, kres_wave);
                            else fill_pass<IO, D, RB, WAVES, NT, false>(p, Xs[1], Xnext, 1, xfirst, g, 1, tile_begins, tile_ends[1], lane, wave, c1, zlds, s_g[1], kq, kres_wave);
                        }
                        have_first = next_too;
                    }
                    if (it == p.iters) { if (side == 0) unit_k = fill; else unit_q = fill; }
                    bool alive;
                    if (side == 0 && it == p.iters) {
                        // The last key pass also contracts with V.  (Its own copy of the exchange, with the
                        // constant true: the other copy then does not keep the 64 registers of U alive.)
#pragma unroll
                        for (int mb = 0; mb < RB; ++mb)
#pragma unroll
                            for (int nb = 0; nb < NB; ++nb)
#pragma unroll
                                for (int j = 0; j < 16; ++j) U[mb][nb][j] = 0.f;
                        // (a SIMD and its 512 registers to itself: three tiles' value rows in flight; otherwise one)
                        accum_from_kept<IO, D, RB, WAVES, NT, (WAVES == 4 && NT >= 8 ? LOT_ACCUM_AHEAD : 1), MASS>(
                            p, reinterpret_cast<const IO*>(p.V), g, tile_begins[0], tile_ends[0], lane, wave,
                            s_v[0], &s_vhl[0][0][0], fill, cs, U, block, nmass[0]);
                        alive = exchange(0, it, true, 1, it - 1, false, !fill);
                    } else {
                        if (side == 0) cheap_pass<IO, RB, WAVES, NT, true, MASS>(p, 0, tile_begins[0], tile_ends[0], lane, wave, s_v[0], &s_vhl[0][0][0], fill, cs, kq, kres_wave, nmass[0]);
                        else cheap_pass<IO, RB, WAVES, NT, false, MASS>(p, 1, tile_begins[1], tile_ends[1], lane, wave, s_v[1], &s_vhl[1][0][0], fill, cs, kq, kres_wave, nmass[1]);
                        alive = exchange(side, it, false, side ^ 1, side == 1 ? it : it - 1, side == 1 && it == p.iters, !fill);
                    }
                    if (!alive) {
                        poison_rows<IO, D>(p, g, tile_begins[1], tile_ends[1], kThreads);
                        return;
                    }
                }
            }
        } else {
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
                if (!exchange(side, it, with_u, side ^ 1, side == 1 ? it : it - 1, side == 1 && it == p.iters, false)) {
                    poison_rows<IO, D>(p, g, tile_begins[1], tile_ends[1], kThreads);
                    return;
                }
            }
        }
        }
        if (attention && p.cluster > 1) {
            // The U partials were posted a whole pass ago: this runs before the last column sums are
            // collected, whose polls are already in flight.
            if (!reduce_u_slice()) { poison_rows<IO, D>(p, g, tile_begins[1], tile_ends[1], kThreads); return; }
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
            // (NT > 0: the passes over the kept kernel matrix leave the factors v_t of both sides to this point)
            auto kept_scale = [&](int t) -> float {
                if constexpr (NT > 0) return (unit_k ? 1.f : s_v[0][t]) * (unit_q ? 1.f : s_v[1][t]);
                else return 1.f;
            };
            if (p.cluster == 1) {
                for (int e = wave * 64 + fresh_lane(); e < 64 * D; e += kThreads) s_u[e] *= s_csinv[e / D] * ((float)p.n_side[1] * s_rho[1][e / D]) * kept_scale(e / D);
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
                    const float sc = s_csinv[e / D] * ((float)p.n_side[1] * s_rho[1][e / D]) * kept_scale(e / D);
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
            if constexpr (NT > 0)
                expand_from_kept<IO, D, RB, WAVES, NT>(p, g, tile_begins[1], tile_ends[1], lane, wave, s_v[1], unit_q, kq, yf_hi, yf_lo,
                                                       reinterpret_cast<IO*>(p.out));
            else
                run_pass<IO, D, RB, EPI_EXPAND, WAVES>(p, Xs[1], nullptr, 1, xfirst, mfirst, g, 1, tile_begins, tile_ends[1], lane, wave, c1, zf, s_zf, s_g[1], cs,
                                                nullptr, U, tr_hi, tr_lo, yf_hi, yf_lo, reinterpret_cast<IO*>(p.out));
        }
        LOT_STAMP(5);
#ifdef LOT_TRACE
        if (threadIdx.x == 0 && p.trace) p.trace[(size_t)blockIdx.x * 128 + 6] = clock64() - clk0;
#endif
#ifdef LOT_TRACE
        if (threadIdx.x == 0 && p.trace) p.trace[(size_t)blockIdx.x * 128 + 7] = valid_a;
#endif
        __syncthreads();   // LDS is reused by the next item
    }
}

// Workgroups the device holds at once for this variant (asked once per device and variant).
template <typename IO, int D, int RB, int WAVES, int NT, bool MASS = false>
int fused_capacity(int* out)
{
    static thread_local int capacity_cache[8] = {0};   // per device ordinal
    int dev = 0;
    LOT_HIP_CHECK(hipGetDevice(&dev));
    int capacity = (dev >= 0 && dev < 8) ? capacity_cache[dev] : 0;
    if (capacity == 0) {
        int per_cu = 0, cus = 0;
        LOT_HIP_CHECK(hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, lot_fused_kernel<IO, D, RB, WAVES, NT, MASS>, WAVES * 64, 0));
        LOT_HIP_CHECK(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev));
        capacity = per_cu * cus;
        if (capacity < 1) { last_hip_error() = hipErrorLaunchOutOfResources; return LOT_ERR_HIP; }
        if (capacity > max_resident_wgs()) capacity = max_resident_wgs();
        if (dev >= 0 && dev < 8) capacity_cache[dev] = capacity;
    }
    *out = capacity;
    return LOT_OK;
}

// Workgroups per problem and tiles per workgroup for a device that holds `capacity` workgroups of
// WAVES wavefronts at once.
struct FusedSplit { int cluster, tiles_per_wg; };
inline FusedSplit fused_split(const Args& a, int waves, int capacity)
{
    const lot_shape& s = a.s;
    const int G = s.B * s.H;
    const int n_side[2] = {a.n_k > 0 ? a.n_k : s.n, a.n_q > 0 ? a.n_q : s.n};
    const int nt_side[2] = {(n_side[0] + kTileTokens - 1) / kTileTokens, (n_side[1] + kTileTokens - 1) / kTileTokens};
    const int ntiles = nt_side[0] > nt_side[1] ? nt_side[0] : nt_side[1];
    int cluster = fused_cluster_bound(s);
    {
        const int by_tiles = (ntiles + waves - 1) / waves;   // at least one tile per wavefront
        if (cluster > by_tiles) cluster = by_tiles;
    }
    if (cluster > capacity / G) cluster = capacity / G;
    if (cluster < 1) cluster = 1;
    FusedSplit sp;
    sp.tiles_per_wg = (ntiles + cluster - 1) / cluster;
    sp.cluster = (ntiles + sp.tiles_per_wg - 1) / sp.tiles_per_wg;
    return sp;
}

// NT > 0: the variant that keeps the kernel matrix on chip; the caller has checked that no wavefront
// gets more than NT tiles of a side (LOT_ERR_PATH otherwise); MASS: the instantiation that takes token masses.
template <typename IO, int D, int RB, int WAVES, int NT, bool MASS = false>
int launch(const Args& a, bool want_out)
{
    constexpr int kThreads = WAVES * 64;
    const lot_shape& s = a.s;
    const int G = s.B * s.H;
    auto kernel = lot_fused_kernel<IO, D, RB, WAVES, NT, MASS>;
    int capacity = 0;
    {
        const int rc = fused_capacity<IO, D, RB, WAVES, NT, MASS>(&capacity);
        if (rc != LOT_OK) return rc;
    }

    // per side: 0 = keys and values, 1 = queries; equal unless this is cross attention
    const int n_side[2] = {a.n_k > 0 ? a.n_k : s.n, a.n_q > 0 ? a.n_q : s.n};
    const int nt_side[2] = {(n_side[0] + kTileTokens - 1) / kTileTokens, (n_side[1] + kTileTokens - 1) / kTileTokens};
    const FusedSplit split = fused_split(a, WAVES, capacity);
    const int cluster = split.cluster;
    if (NT > 0) {
        if ((split.tiles_per_wg + WAVES - 1) / WAVES > NT || !want_out || ((a.mass_q != nullptr || a.mass_k != nullptr) && !MASS))
            return LOT_ERR_PATH;
    }

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
    p.drift_half = 0.5f * drift_limit();
#ifdef LOT_TRACE
    // developer builds: 128 stamps of 8 bytes per workgroup right behind the fused kernel's regions (the
    // caller of such a build allocates 8 MiB more than lot_workspace_bytes says)
    p.trace = (unsigned long long*)(a.ws + a.lay.fused_total);
#else
    p.trace = nullptr;
#endif

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

    if (a.dry_run) {
        if (a.family_out) *a.family_out = NT > 0 ? LOT_KERNELS_KEPT_WORKGROUP : LOT_KERNELS_STREAMING;
        return LOT_OK;
    }
    const int grid = p.num_items < capacity ? p.num_items : capacity;
    // An ordinary launch: the grid never exceeds the number of workgroups the device can hold at
    // once (occupancy query above), which is what the cross-workgroup waits need, and the waits are
    // bounded in any case.  (A cooperative launch would assert the same thing, but kernel tracing
    // tools do not survive it.)
    kernel<<<dim3(grid), dim3(kThreads), 0, a.stream>>>(p);
    LOT_HIP_CHECK(hipGetLastError());
    return LOT_OK;
}

}  // namespace
}  // namespace lot
