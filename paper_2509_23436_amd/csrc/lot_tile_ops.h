// Tile-level operations shared by the multi-launch ("tiled") kernels: coupling weights of a tile,
// transposition of a tile through LDS, the three MFMA contractions (over tokens, Gram, over pivots),
// layout of a pivot-indexed matrix as MFMA B fragments, and the reduction of accumulators over the
// wavefronts of a workgroup.  Workgroups of these kernels have four wavefronts.
#pragma once
#include "lot_tile.h"

namespace lot {
namespace {

constexpr int kWaves = 4;
constexpr int kThreads = kWaves * 64;

// ---------------------------------------------------------------------------------------------
// tile helpers
// ---------------------------------------------------------------------------------------------
template <typename IO, int D, int RB> struct StashBytes { static constexpr int value = RB * (int)sizeof(Frag<IO, D>) * 64; };

// The pivots of the similarity product in LDS, in a layout private to the three functions below.
// fp32 I/O: as bf16 pieces for six bf16 products per step instead of fp32 MFMAs (3/8 of the matrix-
// pipe cycles, and no registers for the pivots), except where the 1.5 times larger area would cost a
// resident workgroup (d = 64 with two pivot blocks).
template <typename IO, int D, int RB>
constexpr bool pivots_in_pieces() { return io_is_f32<IO>::value && !(D == 64 && RB == 2); }
// (ALLOW = false keeps the plain layout for one operand of one kernel, where LDS is short.)
template <typename IO, int D, int RB, bool ALLOW = true> struct PivotStashBytes {
    static constexpr int value = ALLOW && pivots_in_pieces<IO, D, RB>() ? PieceStashBytes<D, RB>::value : StashBytes<IO, D, RB>::value;
};
template <typename IO, int D, int RB, bool ALLOW = true>
__device__ __forceinline__ void stash_similarity_pivots(void* lds, const Frag<IO, D> (&zf)[RB], int lane)
{
    if constexpr (ALLOW && pivots_in_pieces<IO, D, RB>()) stash_pivot_pieces<D, RB>(lds, zf, lane);
    else stash_pivots<D, RB>(lds, zf, lane);
}
// acc += Z X^T for the tile in xf; skew is an opaque zero that keeps the LDS reads inside the tile loop
template <typename IO, int D, int RB, bool ALLOW = true>
__device__ __forceinline__ void similarity_stashed(f32x16 (&acc)[RB], const void* zstash, const Frag<IO, D>& xf,
                                                   int lane, int skew)
{
    if constexpr (ALLOW && pivots_in_pieces<IO, D, RB>()) {
        similarity_pieces<D, RB>(acc, zstash, xf, lane, skew);
    } else {
        Frag<IO, D> zf[RB];
        fetch_pivots<D, RB>(zf, zstash, lane, skew);
        similarity<D, RB>(acc, zf, xf);
    }
}

// On return acc holds e_it = exp2((C_it + g_t) c1 - m_i) (pivots past r give exactly 0) and w the
// reciprocal of their row sum, so the row-normalised kernel is W_it = acc * w.  pot: LDS, 64 floats.
template <typename IO, int D, int RB>
__device__ __forceinline__ void tile_weights(f32x16 (&acc)[RB], float& w, const void* zstash,
                                             const Frag<IO, D>& xf, const float* pot, int lane, float c1, bool valid)
{
    const int kg = lane >> 5;
    int skew = 0;
    asm volatile("" : "+v"(skew));
    load_pivot_vector<RB>(acc, pot + skew, kg);
    similarity_stashed<IO, D, RB>(acc, zstash, xf, lane, skew);
    float m0 = acc[0][0], m1 = acc[0][1];
#pragma unroll
    for (int mb = 0; mb < RB; ++mb)
#pragma unroll
        for (int j = (mb == 0 ? 2 : 0); j < 16; j += 2) {
            m0 = fmaxf(m0, acc[mb][j]);
            m1 = fmaxf(m1, acc[mb][j + 1]);
        }
    const float mc = pair_max(fmaxf(m0, m1)) * c1;
    float s0 = 0.f, s1 = 0.f;
#pragma unroll
    for (int mb = 0; mb < RB; ++mb)
#pragma unroll
        for (int j = 0; j < 16; j += 2) {
            const float e0 = exp2_fast(fmaf(acc[mb][j], c1, -mc));
            const float e1 = exp2_fast(fmaf(acc[mb][j + 1], c1, -mc));
            acc[mb][j] = e0; acc[mb][j + 1] = e1;
            s0 += e0; s1 += e1;
        }
    w = valid ? rcp_fast(pair_sum(s0 + s1)) : 0.f;
}

// The same from similarities that are already there (c: C_it of the tile, accumulator layout): acc = c + g first.
template <int RB>
__device__ __forceinline__ void tile_weights_from_similarities(f32x16 (&acc)[RB], float& w, const f32x16 (&c)[RB],
                                                               const float* pot, int lane, float c1, bool valid)
{
    const int kg = lane >> 5;
    load_pivot_vector<RB>(acc, pot, kg);
#pragma unroll
    for (int mb = 0; mb < RB; ++mb)
#pragma unroll
        for (int j = 0; j < 16; ++j) acc[mb][j] += c[mb][j];
    float m0 = acc[0][0], m1 = acc[0][1];
#pragma unroll
    for (int mb = 0; mb < RB; ++mb)
#pragma unroll
        for (int j = (mb == 0 ? 2 : 0); j < 16; j += 2) {
            m0 = fmaxf(m0, acc[mb][j]);
            m1 = fmaxf(m1, acc[mb][j + 1]);
        }
    const float mc = pair_max(fmaxf(m0, m1)) * c1;
    float s0 = 0.f, s1 = 0.f;
#pragma unroll
    for (int mb = 0; mb < RB; ++mb)
#pragma unroll
        for (int j = 0; j < 16; j += 2) {
            const float e0 = exp2_fast(fmaf(acc[mb][j], c1, -mc));
            const float e1 = exp2_fast(fmaf(acc[mb][j + 1], c1, -mc));
            acc[mb][j] = e0; acc[mb][j + 1] = e1;
            s0 += e0; s1 += e1;
        }
    w = valid ? rcp_fast(pair_sum(s0 + s1)) : 0.f;
}

typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));

// Writes v (accumulator layout, tokens in lanes) transposed into the wavefront's LDS area as bf16
// hi (+ lo when SPLIT), so that rows of 32 tokens can be read back as MFMA operands.  HALF (without
// SPLIT): as fp16 instead -- for values in [0, ~1e4] such as coupling weights it keeps 11 bits where
// bf16 keeps 8, at the same MFMA rate (what falls below its range is far below anything that counts).
template <int RB, bool SPLIT, bool HALF = false>
__device__ __forceinline__ void transpose_tile(const f32x16 (&v)[RB], uint16_t* tr_hi, uint16_t* tr_lo, int i, int kg)
{
    static_assert(!(SPLIT && HALF), "the split form is bf16");
#pragma unroll
    for (int mb = 0; mb < RB; ++mb)
#pragma unroll
        for (int j = 0; j < 16; ++j) {
            const float x = v[mb][j];
            const int pv = pivot_of(mb, j, kg);
            if (HALF) {
                tr_hi[pv * kTrStride + i] = __builtin_bit_cast(uint16_t, (_Float16)x);
            } else {
                const __bf16 h = (__bf16)x;
                tr_hi[pv * kTrStride + i] = __builtin_bit_cast(uint16_t, h);
                if (SPLIT) tr_lo[pv * kTrStride + i] = __builtin_bit_cast(uint16_t, (__bf16)(x - (float)h));
            }
        }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}
__device__ __forceinline__ void transpose_done()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
}

// U[mb][nb] += sum over the tile's tokens of v_it * X_i[NB i' + nb]  (v transposed in LDS; the token
// rows as B fragments vh / vl for the two halves of the tile)
template <int D, int RB, bool SPLIT>
__device__ __forceinline__ void contract_tokens(f32x16 (&U)[RB][D / 32], const uint16_t* tr_hi, const uint16_t* tr_lo,
                                                const bf16x8 (&vh)[2][D / 32], const bf16x8 (&vl)[2][D / 32], int i, int kg)
{
    constexpr int NB = D / 32;
#pragma unroll
    for (int s = 0; s < 2; ++s)
#pragma unroll
        for (int mb = 0; mb < RB; ++mb) {
            const bf16x8 ah = *reinterpret_cast<const bf16x8*>(tr_hi + (32 * mb + i) * kTrStride + 16 * s + 8 * kg);
#pragma unroll
            for (int nb = 0; nb < NB; ++nb) U[mb][nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ah, vh[s][nb], U[mb][nb], 0, 0, 0);
            if (SPLIT) {
                const bf16x8 al = *reinterpret_cast<const bf16x8*>(tr_lo + (32 * mb + i) * kTrStride + 16 * s + 8 * kg);
#pragma unroll
                for (int nb = 0; nb < NB; ++nb) {
                    U[mb][nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(al, vh[s][nb], U[mb][nb], 0, 0, 0);
                    U[mb][nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ah, vl[s][nb], U[mb][nb], 0, 0, 0);
                }
            }
        }
}

// Gm[mb][mb2] += sum over the tile's tokens of v_it v_it'   (t in block mb: registers, t' in block mb2: lanes)
template <int RB, bool SPLIT, bool HALF = false>
__device__ __forceinline__ void contract_gram(f32x16 (&Gm)[RB][RB], const uint16_t* tr_hi, const uint16_t* tr_lo, int i, int kg)
{
    if (HALF) {         // the tile was written as fp16 (transpose_tile<.., HALF = true>)
#pragma unroll
        for (int s = 0; s < 2; ++s) {
            f16x8 a[RB];
#pragma unroll
            for (int mb = 0; mb < RB; ++mb)
                a[mb] = *reinterpret_cast<const f16x8*>(tr_hi + (32 * mb + i) * kTrStride + 16 * s + 8 * kg);
#pragma unroll
            for (int mb = 0; mb < RB; ++mb)
#pragma unroll
                for (int mb2 = mb; mb2 < RB; ++mb2)
                    Gm[mb][mb2] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a[mb], a[mb2], Gm[mb][mb2], 0, 0, 0);
        }
        return;
    }
#pragma unroll
    for (int s = 0; s < 2; ++s) {
        bf16x8 ah[RB], al[RB];
#pragma unroll
        for (int mb = 0; mb < RB; ++mb) {
            ah[mb] = *reinterpret_cast<const bf16x8*>(tr_hi + (32 * mb + i) * kTrStride + 16 * s + 8 * kg);
            if (SPLIT) al[mb] = *reinterpret_cast<const bf16x8*>(tr_lo + (32 * mb + i) * kTrStride + 16 * s + 8 * kg);
        }
#pragma unroll
        for (int mb = 0; mb < RB; ++mb)
#pragma unroll
            for (int mb2 = 0; mb2 < RB; ++mb2) {
                Gm[mb][mb2] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ah[mb], ah[mb2], Gm[mb][mb2], 0, 0, 0);
                if (SPLIT) {
                    Gm[mb][mb2] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(al[mb], ah[mb2], Gm[mb][mb2], 0, 0, 0);
                    Gm[mb][mb2] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ah[mb], al[mb2], Gm[mb][mb2], 0, 0, 0);
                }
            }
    }
}

// out_tile[token][dcol] = sum_t v_it Y_t[dcol]: v in accumulator layout as the A operand, Y as B
// fragments in LDS laid out for the same order of pivots (see lay_out_fragments).
template <int D, int RB, bool SPLIT>
__device__ __forceinline__ void contract_pivots(f32x16 (&o)[D / 32], const f32x16 (&v)[RB],
                                                const bf16x8* yf_hi, const bf16x8* yf_lo, int lane)
{
    constexpr int NB = D / 32;
#pragma unroll
    for (int nb = 0; nb < NB; ++nb)
#pragma unroll
        for (int j = 0; j < 16; ++j) o[nb][j] = 0.f;
#pragma unroll
    for (int s = 0; s < 2 * RB; ++s) {
        f32x8 t;
#pragma unroll
        for (int e = 0; e < 8; ++e) t[e] = v[s >> 1][8 * (s & 1) + e];
        bf16x8 ah, al;
        if (SPLIT) split_bf16(t, ah, al);
        else ah = __builtin_convertvector(t, bf16x8);
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) {
            const bf16x8 yh = yf_hi[(s * NB + nb) * 64 + lane];
            o[nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ah, yh, o[nb], 0, 0, 0);
            if (SPLIT) {
                const bf16x8 yl = yf_lo[(s * NB + nb) * 64 + lane];
                o[nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(al, yh, o[nb], 0, 0, 0);
                o[nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ah, yl, o[nb], 0, 0, 0);
            }
        }
    }
}

// Lays a [64][D] fp32 matrix in LDS (rows = pivots) out as the B fragments contract_pivots reads.
template <int D, int RB>
__device__ __forceinline__ void lay_out_fragments(const float* src, bf16x8* yf_hi, bf16x8* yf_lo, int tid)
{
    constexpr int NB = D / 32;
    for (int f = tid; f < 2 * RB * NB * 64; f += kThreads) {
        const int fl = f & 63, fi = fl & 31, fkg = fl >> 5;
        const int snb = f >> 6, s = snb / NB, nb = snb % NB;
        f32x8 t;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const int pv = 32 * (s >> 1) + 16 * (s & 1) + 8 * (e >> 2) + 4 * fkg + (e & 3);
            t[e] = src[pv * D + NB * fi + nb];
        }
        bf16x8 hi, lo;
        split_bf16(t, hi, lo);
        yf_hi[f] = hi;
        yf_lo[f] = lo;
    }
}

// Sum of a 16 RB NB-register accumulator over the workgroup's wavefronts, in wavefront order, into
// buf (LDS, [64][D], element (pivot, NB i + nb)).  Contains barriers: all wavefronts call it.
template <int D, int RB>
__device__ __forceinline__ void sum_over_waves(const f32x16 (&U)[RB][D / 32], float* buf, int wave, int i, int kg)
{
    constexpr int NB = D / 32;
    for (int turn = 0; turn < kWaves; ++turn) {
        if (wave == turn) {
#pragma unroll
            for (int mb = 0; mb < RB; ++mb)
#pragma unroll
                for (int nb = 0; nb < NB; ++nb)
#pragma unroll
                    for (int j = 0; j < 16; ++j) {
                        float* dst = &buf[pivot_of(mb, j, kg) * D + NB * i + nb];
                        *dst = turn == 0 ? U[mb][nb][j] : *dst + U[mb][nb][j];
                    }
        }
        __syncthreads();
    }
}

// Operand fragment of the similarity MFMA from a row of fp32 numbers in LDS (the bf16 variant rounds
// them to bf16: the products they enter are accumulated in fp32 and the rounding, 2^-9 and zero-mean,
// stays well inside the bf16 output bar).
template <int D>
__device__ __forceinline__ void load_pivots_lds(Frag<uint16_t, D>& f, const float* row, int kg)
{
#pragma unroll
    for (int s = 0; s < D / 16; ++s) {
        f32x8 t;
#pragma unroll
        for (int e = 0; e < 8; ++e) t[e] = row[16 * s + 8 * kg + e];
        f.v[s] = __builtin_convertvector(t, bf16x8);
    }
}
// The part of the same row that the bf16 fragment above leaves out: x - bf16(x), again as bf16.  A
// product taken with both fragments carries the row to about 2^-17.
template <int D>
__device__ __forceinline__ void load_pivots_lds_lo(Frag<uint16_t, D>& f, const float* row, int kg)
{
#pragma unroll
    for (int s = 0; s < D / 16; ++s) {
        f32x8 t;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const float x = row[16 * s + 8 * kg + e];
            t[e] = x - (float)(__bf16)x;
        }
        f.v[s] = __builtin_convertvector(t, bf16x8);
    }
}
template <int D>
__device__ __forceinline__ void load_pivots_lds_lo(Frag<float, D>&, const float*, int) {}   // fp32 fragments are exact
template <int D>
__device__ __forceinline__ void load_pivots_lds(Frag<float, D>& f, const float* row, int kg)
{
#pragma unroll
    for (int s = 0; s < D / 2; ++s) f.v[s] = row[kg * (D / 2) + s];
}



}  // namespace
}  // namespace lot
