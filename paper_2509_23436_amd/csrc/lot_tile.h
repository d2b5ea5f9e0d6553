// Device-side building blocks shared by the fused forward kernel and the tiled backward kernels:
// vector types, MFMA operand fragments of a 32-token x 32 RB-pivot tile, cross-lane reductions,
// agent-coherent loads and stores, barriers.  Everything is inlined; no state.
#pragma once
#include <cmath>

#include "lot_internal.h"

namespace lot {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));

// Pointers that reach the kernel inside the parameter block are generic; loads through them
// become flat instructions, which also count as LDS traffic and defeat the prefetch.  Every
// tensor is device memory, so the accesses are made through explicitly global pointers.
#define LOT_GLOBAL __attribute__((address_space(1)))
template <typename T> __device__ __forceinline__ const LOT_GLOBAL T* as_global(const T* p)
{
    return (const LOT_GLOBAL T*)p;
}
template <typename T> __device__ __forceinline__ LOT_GLOBAL T* as_global(T* p) { return (LOT_GLOBAL T*)p; }

constexpr float kNegBig = -1.0e30f;   // potential of a padding pivot: its exponential is exactly 0
constexpr int kTrStride = 40;         // uint16 per row of the transposed coupling tile (32 + 8 pad)
constexpr float kLog2e = 1.44269504088896340736f;
constexpr float kLn2 = 0.69314718055994530942f;

// ---------------------------------------------------------------------------------------------
// small device helpers
// ---------------------------------------------------------------------------------------------
__device__ __forceinline__ float exp2_fast(float x) { return __builtin_amdgcn_exp2f(x); }
__device__ __forceinline__ float rcp_fast(float x) { return __builtin_amdgcn_rcpf(x); }

// Combine a value with the one held by the lane 32 away (same token, other half of the pivots).
// v_permlane32_swap with both operands equal to x leaves x[lane % 32] in the first result and
// x[32 + lane % 32] in the second, in every lane.  The results are copied to scalars before the
// bit cast: casting the vector elements in place reads the first element twice with this compiler.
__device__ __forceinline__ void both_halves(float x, float& lo, float& hi)
{
    const unsigned u = __builtin_bit_cast(unsigned, x);
    auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
    const unsigned r0 = r[0], r1 = r[1];
    lo = __builtin_bit_cast(float, r0);
    hi = __builtin_bit_cast(float, r1);
}
__device__ __forceinline__ float pair_max(float x)
{
    float lo, hi;
    both_halves(x, lo, hi);
    return fmaxf(lo, hi);
}
__device__ __forceinline__ float pair_sum(float x)
{
    float lo, hi;
    both_halves(x, lo, hi);
    return lo + hi;
}

// The lane index, materialised on the spot.  Code that runs once per pass on one wavefront derives its
// addresses from this instead of from values hoisted out of the iteration loop: under the register
// pressure of the passes those hoisted values are spilled, and every reload from scratch memory costs
// a full memory round trip on the critical path of the exchange.
__device__ __forceinline__ int fresh_lane()
{
    int l;
    asm volatile("v_mbcnt_lo_u32_b32 %0, -1, 0\n\tv_mbcnt_hi_u32_b32 %0, -1, %0" : "=v"(l));
    return l;
}
__device__ __forceinline__ int opaque_scalar(int x)
{
    asm volatile("" : "+s"(x));
    return x;
}

// Workgroup barrier after which one thread may announce, with a relaxed atomic, what the workgroup
// has just stored to global memory.  Every wavefront first waits until its own stores have been
// acknowledged: __syncthreads() alone does not do that (a workgroup-scope release needs no such wait
// on this target, the workgroup shares one L1), and an announcement that overtakes the data lets
// another workgroup read what an earlier launch left at the same address.  The stores themselves
// are write-through (sc1), so the acknowledgement means they have reached the level that agent-
// scope loads read from; no cache write-back is needed.
__device__ __forceinline__ void publish_barrier()
{
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
}

// Workgroup barrier that orders LDS traffic only: nothing here waits for the global loads that
// are in flight for the next tiles.
__device__ __forceinline__ void lds_barrier()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

template <int CTRL> __device__ __forceinline__ float dpp_move(float x)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), CTRL, 0xf, 0xf, true));
}
// Transposing reduction over the 32 lanes that share (lane >> 5).  Every lane comes in with N partial
// sums c[0..N) (one per pivot it covers) and leaves with ONE total: the sum over the 32 lanes of
// c[q], where q = lane % 32 for N = 32 and q = (lane % 32) / 2 for N = 16.  Each step pairs lanes,
// keeps half of the registers and adds the partner's copy of the kept half, so the work halves from
// step to step (about 2 N operations instead of 5 N for N separate butterfly sums).
//   step 1  lane ^ 16   v_permlane16_swap exchanges odd rows of one register with even rows of another
//   step 2  lane ^ 8    row rotation by 8, the write limited to lanes 0-7 / 8-15 of a row by the bank mask
//   step 3  7 - lane    mirror within 8 lanes, bank mask again
//   step 4, 5           within a quad, where bank masks cannot tell lanes apart: select, then add
__device__ __forceinline__ float swap16_add(float a, float b)
{
    auto r = __builtin_amdgcn_permlane16_swap(__builtin_bit_cast(unsigned, a), __builtin_bit_cast(unsigned, b), false, false);
    const unsigned r0 = r[0], r1 = r[1];   // copied out before the casts, as for the 32-lane swap above
    return __builtin_bit_cast(float, r0) + __builtin_bit_cast(float, r1);
}
// The s_nop covers the two wait states required between a vector write of a register and its use as
// a DPP source, which the assembler does not insert inside an asm block.
__device__ __forceinline__ float ror8_add(float a, float b)
{
    float r;
    asm("s_nop 1\n\tv_add_f32_dpp %0, %1, %1 row_ror:8 row_mask:0xf bank_mask:0x3\n\t"
        "v_add_f32_dpp %0, %2, %2 row_ror:8 row_mask:0xf bank_mask:0xc" : "=&v"(r) : "v"(a), "v"(b));
    return r;
}
__device__ __forceinline__ float mirror8_add(float a, float b)
{
    float r;
    asm("s_nop 1\n\tv_add_f32_dpp %0, %1, %1 row_half_mirror row_mask:0xf bank_mask:0x5\n\t"
        "v_add_f32_dpp %0, %2, %2 row_half_mirror row_mask:0xf bank_mask:0xa" : "=&v"(r) : "v"(a), "v"(b));
    return r;
}
template <int CTRL> __device__ __forceinline__ float quad_add(float a, float b, bool upper)
{
    const float keep = upper ? b : a, give = upper ? a : b;
    return keep + dpp_move<CTRL>(give);
}
template <int N> __device__ __forceinline__ float reduce_scatter_tokens(float (&c)[N], int i)
{
    static_assert(N == 32 || N == 16, "16 accumulator registers per block of 32 pivots");
#pragma unroll
    for (int q = 0; q < N / 2; ++q) c[q] = swap16_add(c[q], c[q + N / 2]);
#pragma unroll
    for (int q = 0; q < N / 4; ++q) c[q] = ror8_add(c[q], c[q + N / 4]);
#pragma unroll
    for (int q = 0; q < N / 8; ++q) c[q] = mirror8_add(c[q], c[q + N / 8]);
#pragma unroll
    for (int q = 0; q < N / 16; ++q) c[q] = quad_add<0x4E>(c[q], c[q + N / 16], (i & 2) != 0);   // quad_perm [2,3,0,1]
    if (N == 32) return quad_add<0xB1>(c[0], c[1], (i & 1) != 0);                                // quad_perm [1,0,3,2]
    return c[0] + dpp_move<0xB1>(c[0]);
}

// Agent-coherent loads that the compiler can schedule: raw buffer loads carrying the sc1 cache
// policy (the same policy an agent-scope atomic load uses).  An atomic load written in C++ is
// followed by a full wait each time, which turns a gather of k partial results into k sequential
// round trips to memory; these are tracked like ordinary loads, so several can be in flight and
// other work can be placed between issue and first use.
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
constexpr int kCoherent = 16;   // cache-policy operand: sc1
__device__ __forceinline__ __amdgpu_buffer_rsrc_t coherent_view(const void* base)
{
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), 0, 0x7fffffff, 0x00020000);
}
__device__ __forceinline__ float ldc_f32(__amdgpu_buffer_rsrc_t v, uint32_t byte_offset)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(v, byte_offset, 0, kCoherent));
}
__device__ __forceinline__ unsigned long long ldc_u64(__amdgpu_buffer_rsrc_t v, uint32_t byte_offset)
{
    const u32x2 w = __builtin_amdgcn_raw_buffer_load_b64(v, byte_offset, 0, kCoherent);
    return ((unsigned long long)w[1] << 32) | (unsigned long long)w[0];
}
__device__ __forceinline__ f32x4 ldc_f32x4(__amdgpu_buffer_rsrc_t v, uint32_t byte_offset)
{
    return __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(v, byte_offset, 0, kCoherent));
}
__device__ __forceinline__ void st_coherent(float* p, float v)
{
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Bounded waits between workgroups: the status words of a workspace ([0] = nonce of a launch in which a wait
// gave up) and a poll with a budget.
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

__device__ __forceinline__ void split_bf16(const f32x8& x, bf16x8& hi, bf16x8& lo)
{
    hi = __builtin_convertvector(x, bf16x8);
    const f32x8 back = __builtin_convertvector(hi, f32x8);
    lo = __builtin_convertvector(x - back, bf16x8);
}
__device__ __forceinline__ uint16_t bf16_bits_of(float x) { return __builtin_bit_cast(uint16_t, (__bf16)x); }

// Cross-workgroup exchange protocol.  Every word that one workgroup writes and another reads
// (partial sums, the Y tile, the counters) is accessed ONLY with agent-scope relaxed atomics, which
// go to the device-wide coherence point.  Ordering comes from the workgroup barrier: it waits until
// the writers' stores have been acknowledged before thread 0 bumps the counter, and the readers load
// after thread 0 has seen the counter.  No agent-scope release/acquire fence is used on purpose:
// on this multi-die part such a fence writes back / invalidates a whole L2, once per workgroup per
// iteration, which costs far more than the iteration itself.
//
// ---------------------------------------------------------------------------------------------
// operand fragments of the similarity MFMA
// ---------------------------------------------------------------------------------------------
// bf16: v_mfma_f32_32x32x16_bf16, lane (i = lane % 32, kg = lane / 32) supplies, for step s,
//       elements [16 s + 8 kg, +8) of row i.                       D/16 steps.
// fp32: v_mfma_f32_32x32x2_f32, lane supplies element kg*(D/2) + s. D/2 steps.  The same registers
//       also feed the bf16-piece form of the product (similarity_pieces below): registers
//       [8 s, 8 s + 8) of a lane are then its eight numbers of bf16 step s, D/16 steps.
template <typename IO, int D> struct Frag;
template <int D> struct Frag<uint16_t, D> { bf16x8 v[D / 16]; };
template <int D> struct Frag<float, D> { float v[D / 2]; };

template <int D>
__device__ __forceinline__ void load_tokens(Frag<uint16_t, D>& f, const uint16_t* row, int kg)
{
#pragma unroll
    for (int s = 0; s < D / 16; ++s) f.v[s] = *as_global(reinterpret_cast<const bf16x8*>(row + 16 * s + 8 * kg));
}
template <int D>
__device__ __forceinline__ void load_tokens(Frag<float, D>& f, const float* row, int kg)
{
#pragma unroll
    for (int q = 0; q < D / 8; ++q) {
        const f32x4 t = *as_global(reinterpret_cast<const f32x4*>(row + kg * (D / 2) + 4 * q));
#pragma unroll
        for (int e = 0; e < 4; ++e) f.v[4 * q + e] = t[e];
    }
}

// pivot rows: Z is fp32 in memory; the bf16 path rounds it to bf16 (nearest even) here.
// zrow always points at a real row (the caller clamps the index), so the loads are unconditional
// 16-byte vectors; rows of padding pivots are zeroed afterwards.
template <int D>
__device__ __forceinline__ void load_pivots(Frag<uint16_t, D>& f, const float* zrow, int kg, bool valid)
{
    f32x4 raw[D / 16][2];
#pragma unroll
    for (int s = 0; s < D / 16; ++s)
#pragma unroll
        for (int q = 0; q < 2; ++q) raw[s][q] = *as_global(reinterpret_cast<const f32x4*>(zrow + 16 * s + 8 * kg + 4 * q));
#pragma unroll
    for (int s = 0; s < D / 16; ++s) {
        f32x8 t;
#pragma unroll
        for (int e = 0; e < 8; ++e) t[e] = valid ? raw[s][e >> 2][e & 3] : 0.f;
        f.v[s] = __builtin_convertvector(t, bf16x8);
    }
}
template <int D>
__device__ __forceinline__ void load_pivots(Frag<float, D>& f, const float* zrow, int kg, bool valid)
{
    f32x4 raw[D / 8];
#pragma unroll
    for (int q = 0; q < D / 8; ++q) raw[q] = *as_global(reinterpret_cast<const f32x4*>(zrow + kg * (D / 2) + 4 * q));
#pragma unroll
    for (int s = 0; s < D / 2; ++s) f.v[s] = valid ? raw[s >> 2][s & 3] : 0.f;
}

// Pivot fragments kept in LDS as [block][step][lane], so that the heavier passes need not hold
// them in registers.  `skew` is an opaque zero that keeps the loads inside the tile loop.
template <int D, int RB>
__device__ __forceinline__ void stash_pivots(void* lds, const Frag<uint16_t, D> (&zf)[RB], int lane)
{
    bf16x8* dst = reinterpret_cast<bf16x8*>(lds);
#pragma unroll
    for (int mb = 0; mb < RB; ++mb)
#pragma unroll
        for (int s = 0; s < D / 16; ++s) dst[(mb * (D / 16) + s) * 64 + lane] = zf[mb].v[s];
}
template <int D, int RB>
__device__ __forceinline__ void stash_pivots(void* lds, const Frag<float, D> (&zf)[RB], int lane)
{
    float* dst = reinterpret_cast<float*>(lds);
#pragma unroll
    for (int mb = 0; mb < RB; ++mb)
#pragma unroll
        for (int s = 0; s < D / 2; ++s) dst[(mb * (D / 2) + s) * 64 + lane] = zf[mb].v[s];
}
template <int D, int RB>
__device__ __forceinline__ void fetch_pivots(Frag<uint16_t, D> (&zf)[RB], const void* lds, int lane, int skew)
{
    const bf16x8* src = reinterpret_cast<const bf16x8*>(lds) + skew;
#pragma unroll
    for (int mb = 0; mb < RB; ++mb)
#pragma unroll
        for (int s = 0; s < D / 16; ++s) zf[mb].v[s] = src[(mb * (D / 16) + s) * 64 + lane];
}
template <int D, int RB>
__device__ __forceinline__ void fetch_pivots(Frag<float, D> (&zf)[RB], const void* lds, int lane, int skew)
{
    const float* src = reinterpret_cast<const float*>(lds) + skew;
#pragma unroll
    for (int mb = 0; mb < RB; ++mb)
#pragma unroll
        for (int s = 0; s < D / 2; ++s) zf[mb].v[s] = src[(mb * (D / 2) + s) * 64 + lane];
}

// acc[mb] += Z_block(mb) X_tile^T   (pivots x tokens); acc enters holding the pivot potentials
// Eight fp32 numbers as three bf16 vectors whose sum is exact: h = the upper 16 bits, m = the upper
// 16 bits of what is left, l = the rest (at most 8 significant bits by then).
struct Pieces { bf16x8 h, m, l; };
__device__ __forceinline__ void cut_in_three(const float* v, Pieces& out)
{
    typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
    u32x4 ph, pm, pl;
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        uint32_t hb[2], mbits[2], lb[2];
#pragma unroll
        for (int e = 0; e < 2; ++e) {
            const float x = v[2 * u + e];
            hb[e] = __builtin_bit_cast(uint32_t, x);
            const float r1 = x - __builtin_bit_cast(float, hb[e] & 0xffff0000u);
            mbits[e] = __builtin_bit_cast(uint32_t, r1);
            const float r2 = r1 - __builtin_bit_cast(float, mbits[e] & 0xffff0000u);
            lb[e] = __builtin_bit_cast(uint32_t, r2);
        }
        // upper halves of the two words, the first in the low half of the result
        ph[u] = __builtin_amdgcn_perm(hb[1], hb[0], 0x07060302u);
        pm[u] = __builtin_amdgcn_perm(mbits[1], mbits[0], 0x07060302u);
        pl[u] = __builtin_amdgcn_perm(lb[1], lb[0], 0x07060302u);
    }
    out.h = __builtin_bit_cast(bf16x8, ph);
    out.m = __builtin_bit_cast(bf16x8, pm);
    out.l = __builtin_bit_cast(bf16x8, pl);
}

template <int D, int RB>
__device__ __forceinline__ void similarity(f32x16 (&acc)[RB], const Frag<uint16_t, D> (&zf)[RB],
                                           const Frag<uint16_t, D>& xf)
{
#pragma unroll
    for (int s = 0; s < D / 16; ++s)
#pragma unroll
        for (int mb = 0; mb < RB; ++mb)
            acc[mb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(zf[mb].v[s], xf.v[s], acc[mb], 0, 0, 0);
}
template <int D, int RB>
__device__ __forceinline__ void similarity(f32x16 (&acc)[RB], const Frag<float, D> (&zf)[RB],
                                           const Frag<float, D>& xf)
{
#pragma unroll
    for (int s = 0; s < D / 2; ++s)
#pragma unroll
        for (int mb = 0; mb < RB; ++mb)
            acc[mb] = __builtin_amdgcn_mfma_f32_32x32x2f32(zf[mb].v[s], xf.v[s], acc[mb], 0, 0, 0);
}

// The same product with the fp32 operands as three bf16 pieces each (8 + 8 + 8 significant bits, cut,
// not rounded, so the pieces add up to the number exactly) and the six products that matter: what is
// left out is below 2^-23 of |z||x|, and six bf16 products cost 3/8 of the matrix-pipe cycles of the
// fp32 MFMA.  The contraction index may be permuted freely as long as both operands agree: a lane's
// eight consecutive registers are taken as its eight numbers of one MFMA step.  The pivots' pieces are
// cut once and kept in LDS ([block][step][piece][lane] vectors of 8); the token rows are cut here.
template <int D, int RB> struct PieceStashBytes { static constexpr int value = RB * (D / 16) * 3 * 64 * 16; };
template <int D, int RB>
__device__ __forceinline__ void stash_pivot_pieces(void* lds, const Frag<float, D> (&zf)[RB], int lane)
{
    bf16x8* dst = reinterpret_cast<bf16x8*>(lds);
#pragma unroll
    for (int mb = 0; mb < RB; ++mb)
#pragma unroll
        for (int s = 0; s < D / 16; ++s) {
            Pieces zp;
            cut_in_three(zf[mb].v + 8 * s, zp);
            bf16x8* at = dst + (size_t)((mb * (D / 16) + s) * 3) * 64 + lane;
            at[0] = zp.h; at[64] = zp.m; at[128] = zp.l;
        }
}
template <int D, int RB>
__device__ __forceinline__ void similarity_pieces(f32x16 (&acc)[RB], const void* lds, const Frag<float, D>& xf,
                                                  int lane, int skew)
{
    const bf16x8* src = reinterpret_cast<const bf16x8*>(lds) + skew;
#pragma unroll
    for (int s = 0; s < D / 16; ++s) {
        Pieces xp;
        cut_in_three(xf.v + 8 * s, xp);
#pragma unroll
        for (int mb = 0; mb < RB; ++mb) {
            const bf16x8* at = src + (size_t)((mb * (D / 16) + s) * 3) * 64 + lane;
            const bf16x8 zh = at[0], zm = at[64], zl = at[128];
            acc[mb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(zl, xp.h, acc[mb], 0, 0, 0);
            acc[mb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(zh, xp.l, acc[mb], 0, 0, 0);
            acc[mb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(zm, xp.m, acc[mb], 0, 0, 0);
            acc[mb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(zm, xp.h, acc[mb], 0, 0, 0);
            acc[mb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(zh, xp.m, acc[mb], 0, 0, 0);
            acc[mb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(zh, xp.h, acc[mb], 0, 0, 0);
        }
    }
}

// pivot index of accumulator register j of block mb in lane-half kg
__device__ __forceinline__ int pivot_of(int mb, int j, int kg) { return 32 * mb + 8 * (j >> 2) + 4 * kg + (j & 3); }

// load a per-pivot vector from LDS into accumulator layout
template <int RB>
__device__ __forceinline__ void load_pivot_vector(f32x16 (&dst)[RB], const float* src, int kg)
{
#pragma unroll
    for (int mb = 0; mb < RB; ++mb)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const f32x4 t = *reinterpret_cast<const f32x4*>(src + 32 * mb + 8 * q + 4 * kg);
#pragma unroll
            for (int e = 0; e < 4; ++e) dst[mb][4 * q + e] = t[e];
        }
}

// ---------------------------------------------------------------------------------------------
// values / output element access by I/O type
// ---------------------------------------------------------------------------------------------
// Loads V[token][NB*i + nb], nb < NB, for 8 tokens and returns them as MFMA B fragments (hi, lo).
template <int D>
__device__ __forceinline__ void load_values(bf16x8 (&hi)[D / 32], bf16x8 (&lo)[D / 32], const uint16_t* V,
                                            size_t row0, int n_left, int i)
{
    constexpr int NB = D / 32;
    union { bf16x8 v; uint16_t u[8]; } h[NB];
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        const size_t row = row0 + (e < n_left ? e : n_left - 1);
        if (NB == 2) {
            const uint32_t w = *as_global(reinterpret_cast<const uint32_t*>(V + row * D + 2 * i));
            h[0].u[e] = (uint16_t)(w & 0xffffu);
            h[NB - 1].u[e] = (uint16_t)(w >> 16);
        } else {
            h[0].u[e] = as_global(V)[row * D + i];
        }
    }
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) { hi[nb] = h[nb].v; lo[nb] = h[nb].v; }
}
template <int D>
__device__ __forceinline__ void load_values(bf16x8 (&hi)[D / 32], bf16x8 (&lo)[D / 32], const float* V,
                                            size_t row0, int n_left, int i)
{
    constexpr int NB = D / 32;
    f32x8 t[NB];
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        const size_t row = row0 + (e < n_left ? e : n_left - 1);
        if (NB == 2) {
            const f32x2 w = *as_global(reinterpret_cast<const f32x2*>(V + row * D + 2 * i));
            t[0][e] = w[0];
            t[NB - 1][e] = w[1];
        } else {
            t[0][e] = as_global(V)[row * D + i];
        }
    }
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) split_bf16(t[nb], hi[nb], lo[nb]);
}

// The same in two steps, for passes that keep the value rows of several tiles in flight: the loads leave
// what they fetched untouched (one register per row: two bf16 channels for D = 64, one for D = 32), and the
// operand fragments are formed from those registers only when the tile is multiplied -- formed right behind
// the loads they would make the wavefront wait for the data at once.  `row_of(s, e)` gives the row of
// token e of step s (16 tokens in all), already clamped to the tensor.
template <int D, typename RowOf>
__device__ __forceinline__ void request_value_rows(uint32_t (&raw)[16], const uint16_t* V, int i, RowOf row_of)
{
#pragma unroll
    for (int s = 0; s < 2; ++s)
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const size_t row = row_of(s, e);
            if (D == 64) raw[8 * s + e] = *as_global(reinterpret_cast<const uint32_t*>(V + row * D + 2 * i));
            else raw[8 * s + e] = as_global(V)[row * D + i];
        }
}
// (all 16 rows in range: `base` points at the lane's element of the first row, the others are constant offsets)
template <int D>
__device__ __forceinline__ void request_value_rows_inside(uint32_t (&raw)[16], const uint16_t* base)
{
#pragma unroll
    for (int s = 0; s < 2; ++s)
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            if (D == 64) raw[8 * s + e] = *as_global(reinterpret_cast<const uint32_t*>(base + (16 * s + e) * D));
            else raw[8 * s + e] = as_global(base)[(16 * s + e) * D];
        }
}
template <int D>
__device__ __forceinline__ void value_fragments(bf16x8 (&hi)[2][D / 32], const uint32_t (&raw)[16])
{
#pragma unroll
    for (int s = 0; s < 2; ++s) {
        u32x4 lo16, hi16;
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const uint32_t a = raw[8 * s + 2 * k], b = raw[8 * s + 2 * k + 1];
            lo16[k] = (a & 0xffffu) | (b << 16);
            hi16[k] = (a >> 16) | (b & 0xffff0000u);
        }
        hi[s][0] = __builtin_bit_cast(bf16x8, lo16);
        if (D == 64) hi[s][D / 32 - 1] = __builtin_bit_cast(bf16x8, hi16);
    }
}

template <int NB> __device__ __forceinline__ void store_out(uint16_t* row, int i, float a, float b)
{
    if (NB == 2) *as_global(reinterpret_cast<uint32_t*>(row + 2 * i)) = (uint32_t)bf16_bits_of(a) | ((uint32_t)bf16_bits_of(b) << 16);
    else as_global(row)[i] = bf16_bits_of(a);
}
template <int NB> __device__ __forceinline__ void store_out(float* row, int i, float a, float b)
{
    if (NB == 2) { f32x2 w; w[0] = a; w[1] = b; *as_global(reinterpret_cast<f32x2*>(row + 2 * i)) = w; }
    else as_global(row)[i] = a;
}

template <typename IO> struct io_is_f32 { static constexpr bool value = false; };
template <> struct io_is_f32<float> { static constexpr bool value = true; };

}  // namespace
}  // namespace lot
