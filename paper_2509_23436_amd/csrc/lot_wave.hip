// LOT attention forward for short sequences: one workgroup of two wavefronts per (batch, head) problem,
// wavefront 0 the keys' solve, wavefront 1 the queries' -- or WS = 2 or 4 wavefronts per side, each holding
// NT of the side's tiles, which add up their column sums through local memory once per iteration (the only
// workgroup barrier of an iteration).
//
// A side of at most 32 NT tokens has a kernel matrix exp(C/eps) of NT tiles of 32 tokens x 32 RB
// pivots, which one wavefront can hold in its registers (bf16 pairs for bf16 I/O, fp32 for fp32 I/O;
// one wavefront per SIMD, so the whole register file is its own).  The two Sinkhorn solves of a problem
// are independent until the very end (paper, Method: the two entropic problems share only Z, beta and
// eps), so each wavefront runs all T iterations of its side on its own, in the scaling form the paper
// prints (Gamma = Diag(u) exp(C/eps) Diag(v)): per iteration one sweep over its registers
//     s_i = sum_t Kt_it v_t,   colsum_t = v_t sum_i Kt_it / s_i,   g_t += eps log(n beta_t / colsum_t)
// a reduction over the lanes (one pivot per lane afterwards), the pivot update in that layout, and the
// new v handed back to the tile layout through 256 bytes of LDS.  No workgroup barrier, no global
// memory and no exponential per element inside the iterations; Q and K are read once.  The last key
// sweep also contracts with V (transposing its tiles through LDS, as the fused kernel does); the two
// wavefronts meet once, after which the queries' wavefront expands O = n Gamma1 Diag(beta)^-1 (Gamma2 V).
// As in the fused kernel's kept-matrix variants the potentials may drift from those folded into the
// kept matrix by kDriftLimit / 2 binary orders per pivot before the matrix is recomputed.
#include "lot_fused_kernel.h"

namespace lot {
namespace {

struct WaveParams {
    const void* Q; const void* K; const void* V;
    const float* Z; const float* beta;
    void* out;
    int G, H, r, iters;
    int n_side[2];        // 0 = keys and values, 1 = queries and the output
    int stride_side[2];   // tokens between consecutive problems in memory
    const float* mass_side[2];   // [G][n_side] token masses, or null: uniform 1 / n_side
    unsigned long long* status;  // the workspace's status words: [1] takes the launch's nonce (nothing here can fail,
    unsigned long long nonce;    // and a mark that an earlier, failed launch of another kernel left must not outlive it)
    float eps;
    float drift_half;     // a pivot's potential may move this many binary orders away from pivot 0's before the kernel matrix is recomputed
    unsigned long long* trace;   // LOT_TRACE builds only: 32 stamps for the first wavefront of each side, 128 per workgroup
};

#ifdef LOT_TRACE
#define LOT_WSTAMP(slot) do { if (lane == 0 && part == 0 && p.trace) p.trace[(size_t)blockIdx.x * 128 + side * 32 + (slot)] = wall_clock64(); } while (0)
#else
#define LOT_WSTAMP(slot) do { } while (0)
#endif

// pivot that lane (i, kg) holds after reduce_scatter_tokens<16 RB>
template <int RB> __device__ __forceinline__ int reduced_pivot(int i, int kg)
{
    const int q = RB == 2 ? i : i >> 1;
    return 32 * (q >> 4) + 8 * ((q & 15) >> 2) + 4 * kg + (q & 3);
}

__device__ __forceinline__ void wave_sync_lds()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// WS wavefronts per side (the first WS of the workgroup are the keys'), NT tiles per wavefront; WPE wavefronts
// share a SIMD's registers (1: all 512 for one wavefront; 2: twice as many problems resident).
// One word of every 128-byte line of `bytes` bytes from `base` (at most 64 kLoads lines): the lines are then
// on their way into the caches while the wavefront works on something else, and the loads that later fetch
// the rows find them there.  The words are handed back so that the caller can keep them alive until a point
// where waiting for them costs nothing (a dropped result would let the register be reused while the load is
// still in flight).
template <int kLoads>
__device__ __forceinline__ void touch_lines(uint32_t (&word)[kLoads], const void* base, int bytes, int lane)
{
    const int lines = (bytes + 127) / 128;
#pragma unroll
    for (int k = 0; k < kLoads; ++k) {
        const int line = min(lane + 64 * k, lines - 1);
        word[k] = lines > 0 ? *as_global(reinterpret_cast<const uint32_t*>(static_cast<const char*>(base) + (size_t)line * 128)) : 0u;
    }
}
template <int kLoads> __device__ __forceinline__ void touched(const uint32_t (&word)[kLoads])
{
#pragma unroll
    for (int k = 0; k < kLoads; ++k) asm volatile("" ::"v"(word[k]));
}

template <typename IO, int D, int RB, int NT, int WS, int WPE>
__global__ void __launch_bounds__(128 * WS) __attribute__((amdgpu_waves_per_eu(WPE, WPE))) lot_wave_kernel(WaveParams p)
{
    constexpr int NB = D / 32;
    constexpr int NW = ResWords<IO, RB>::value;
    constexpr bool kSplit = io_is_f32<IO>::value;
    constexpr bool kPieces = io_is_f32<IO>::value;
    __shared__ __attribute__((aligned(16))) float s_vec[2 * WS][64];  // per wavefront: a per-pivot vector on its way into tile layout
    __shared__ __attribute__((aligned(16))) float s_part[WS > 1 ? 2 : 1][2 * WS][64];   // column sums of a side's wavefronts (two parities)
    __shared__ __attribute__((aligned(16))) float s_fac[WS][64];      // keys: v_t / colsum_t, the factor of the rows of U
    __shared__ __attribute__((aligned(16))) float s_qs[64];           // queries: n rho_t v_t
    constexpr int kUBufs = WS < 2 ? WS : 2;
    __shared__ __attribute__((aligned(16))) float s_u[kUBufs][64 * D];   // the key wavefronts' shares of U, scaled to Y' (wavefronts 2, 3 add to 0, 1)
    __shared__ __attribute__((aligned(16))) uint16_t s_tr[WS][2 * 32 * RB * kTrStride];   // keys: transposed tile (hi, lo)
    __shared__ __attribute__((aligned(16))) bf16x8 s_yf[2][2 * RB * NB * 64];         // Y'' as MFMA operand fragments (hi, lo)
    __shared__ __attribute__((aligned(16))) char s_zf[kPieces ? PieceStashBytes<D, RB>::value : 16];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int side = wave / WS, part = wave % WS;                    // side 0: keys, 1: queries
    const int i = lane & 31, kg = lane >> 5;
    const int g = blockIdx.x, h = g % p.H;
    const int r = p.r;
    if (g == 0 && tid == 0) __hip_atomic_store(p.status + 1, p.nonce, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    const int n = p.n_side[side], stride = p.stride_side[side];
    const float c1 = kLog2e / p.eps;
    // this wavefront's tiles: NT consecutive ones from tile part * NT of the side (tok0 = its first token)
    const int tok0 = part * NT * kTileTokens;
    // (none of them below n: an idle wavefront, which still takes part in every barrier; token indices are
    // clamped to n - 1 wherever they form an address)
    const IO* X = reinterpret_cast<const IO*>(side == 0 ? p.K : p.Q) + (size_t)g * stride * D;
    const int ntiles = max(0, min((n + kTileTokens - 1) / kTileTokens - part * NT, NT));

    LOT_WSTAMP(0);
    // ---- pivots: operand fragments, needed only where the kernel matrix is computed (loaded there: held in
    //      registers through the iterations they would only take room)
    auto load_all_pivots = [&](Frag<IO, D> (&zf)[RB]) __attribute__((always_inline)) {
#pragma unroll
        for (int mb = 0; mb < RB; ++mb) {
            const int t = 32 * mb + i;
            load_pivots<D>(zf[mb], p.Z + ((size_t)h * r + min(t, r - 1)) * D, kg, t < r);
        }
    };
#ifdef LOT_TRACE
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    LOT_WSTAMP(21);
#endif
    // the first tile's rows
    Frag<IO, D> xc;
    load_tokens<D>(xc, X + (size_t)min(tok0 + i, n - 1) * D, kg);
    // the rows of the tiles that the first pass does not request at once (it keeps kAhead tiles in flight) and,
    // on the keys' side, the value rows of the last sweep: touched now, so that they stream in from memory
    // while the first tiles and the iterations are worked on
    constexpr int kAheadMax = 4;
    constexpr int kAhead = NT < kAheadMax ? NT : kAheadMax;
    constexpr int kRowBytes = D * (int)sizeof(IO);
    constexpr int kTouchX = NT > kAhead ? ((NT - kAhead) * kTileTokens * kRowBytes / 128 + 63) / 64 : 1;
    constexpr int kTouchV = (NT * kTileTokens * kRowBytes / 128 + 63) / 64;
    uint32_t touch_x[kTouchX], touch_v[kTouchV];
#pragma unroll
    for (int k = 0; k < kTouchV; ++k) touch_v[k] = 0u;
    {
        const int first = tok0 + kAhead * kTileTokens, last = min(n, tok0 + NT * kTileTokens);
        touch_lines<kTouchX>(touch_x, X + (size_t)min(first, n - 1) * D, NT > kAhead ? max(last - first, 0) * kRowBytes : 0, lane);
    }
#ifdef LOT_TRACE
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    LOT_WSTAMP(22);
#endif
    // this lane's pivot in the layout the column sums are reduced to
    const int piv = reduced_pivot<RB>(i, kg);
    const bool live = piv < r;
    const float beta_l = as_global(p.beta)[(size_t)h * r + min(piv, r - 1)];
    const float nbeta = (float)n * beta_l;
    float g_l = 0.f, gref_l = 0.f;        // this pivot's potential, and the one folded into the kept matrix
    if constexpr (kPieces) {
        if (wave == 0) {
            Frag<IO, D> zf[RB];
            load_all_pivots(zf);
            stash_pivot_pieces<D, RB>(s_zf, zf, lane);
        }
        __syncthreads();
    }

    uint32_t kq[NT][NW];
#pragma unroll
    for (int sl = 0; sl < NT; ++sl)
#pragma unroll
        for (int q = 0; q < NW; ++q) kq[sl][q] = 0u;
    // token masses times n (1 for uniform masses): they weight what a token adds to the column sums and to the
    // contraction with V, not its own row of the output (paper, "Empirical measures and pivot": general marginals)
    float nm[NT];
    {
        const float* const mass = p.mass_side[side];
#pragma unroll
        for (int sl = 0; sl < NT; ++sl) {
            const int tok = tok0 + sl * kTileTokens + i;
            nm[sl] = (mass != nullptr && tok < n) ? (float)n * as_global(mass)[(size_t)g * n + tok] : 1.f;
        }
    }

    // ---- the kernel matrix with the current potentials folded in (zero at first; -big for padding pivots).
    //      A single wavefront per SIMD has nobody to switch to while it waits for memory, so the rows of
    //      kAhead tiles are kept in flight.
    auto fill = [&](bool first) __attribute__((always_inline)) {
        Frag<IO, D> zf[RB];
        if constexpr (!kPieces) load_all_pivots(zf);
        f32x16 gv[RB];
        s_vec[wave][piv] = live ? g_l : kNegBig;
        wave_sync_lds();
        load_pivot_vector<RB>(gv, s_vec[wave], kg);
        wave_sync_lds();
        if (first) LOT_WSTAMP(20);
        // (addresses are formed from a lane index that the compiler cannot see through: hoisted out of the
        // iteration loop, the addresses of all slots would be hundreds of live registers)
        int io = i;
        asm volatile("" : "+v"(io));
        Frag<IO, D> xs[kAhead];
#pragma unroll
        for (int a = 0; a < kAhead; ++a) {
            if (a == 0 && first) xs[0] = xc;      // (requested before the pivots were loaded)
            else if (a < ntiles) load_tokens<D>(xs[a], X + (size_t)min(tok0 + a * kTileTokens + io, n - 1) * D, kg);
        }
#pragma unroll
        for (int slot = 0; slot < NT; ++slot) {
            if (slot < ntiles) {
                f32x16 acc[RB];
#pragma unroll
                for (int mb = 0; mb < RB; ++mb) acc[mb] = gv[mb];
                if constexpr (kPieces) similarity_pieces<D, RB>(acc, s_zf, xs[slot % kAhead], lane, 0);
                else similarity<D, RB>(acc, zf, xs[slot % kAhead]);
                if (slot + kAhead < NT) {
                    if (slot + kAhead < ntiles)
                        load_tokens<D>(xs[slot % kAhead], X + (size_t)min(tok0 + (slot + kAhead) * kTileTokens + io, n - 1) * D, kg);
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
                res_pack<IO, RB>(kq[slot], acc);
                if (first) LOT_WSTAMP(12 + slot);
            }
            __builtin_amdgcn_sched_barrier(0);   // (slots are not interleaved: that would only cost registers)
        }
        gref_l = g_l;
    };

    f32x16 vC[RB];                       // v in tile layout
    float v_l = 1.f;                     // this lane's pivot's v
    float rho_l = 0.f;                   // after the last iteration: beta_t / colsum_t (queries), 1 / colsum_t (keys)

    // one sweep over the kept matrix: column sums of Kt_it / s_i (the factor v_t is applied afterwards)
    auto sweep = [&](f32x16 (&cs)[RB]) __attribute__((always_inline)) {
#pragma unroll
        for (int mb = 0; mb < RB; ++mb)
#pragma unroll
            for (int j = 0; j < 16; ++j) cs[mb][j] = 0.f;
#pragma unroll
        for (int slot = 0; slot < NT; ++slot) {
            if (slot < ntiles) {
                f32x16 k[RB];
                res_unpack<IO, RB>(k, kq[slot]);
                float s0 = 0.f, s1 = 0.f, s2 = 0.f, s3 = 0.f;
#pragma unroll
                for (int mb = 0; mb < RB; ++mb)
#pragma unroll
                    for (int j = 0; j < 16; j += 4) {
                        s0 = fmaf(k[mb][j], vC[mb][j], s0);
                        s1 = fmaf(k[mb][j + 1], vC[mb][j + 1], s1);
                        s2 = fmaf(k[mb][j + 2], vC[mb][j + 2], s2);
                        s3 = fmaf(k[mb][j + 3], vC[mb][j + 3], s3);
                    }
                const float s = pair_sum((s0 + s1) + (s2 + s3));
                const float w = tok0 + slot * kTileTokens + i < n ? rcp_fast(s) * nm[slot] : 0.f;
#pragma unroll
                for (int mb = 0; mb < RB; ++mb)
#pragma unroll
                    for (int j = 0; j < 16; ++j) cs[mb][j] = fmaf(k[mb][j], w, cs[mb][j]);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
    };

    // the same sweep for the keys' last iteration: also U = sum_j (Kt_jt / s_j) V_j
    f32x16 U[RB][NB];
    auto sweep_with_values = [&](f32x16 (&cs)[RB]) __attribute__((always_inline)) {
        const IO* V = reinterpret_cast<const IO*>(p.V);
        uint16_t* tr_hi = s_tr[part];
        uint16_t* tr_lo = s_tr[part] + 32 * RB * kTrStride;
#pragma unroll
        for (int mb = 0; mb < RB; ++mb) {
#pragma unroll
            for (int j = 0; j < 16; ++j) cs[mb][j] = 0.f;
#pragma unroll
            for (int nb = 0; nb < NB; ++nb)
#pragma unroll
                for (int j = 0; j < 16; ++j) U[mb][nb][j] = 0.f;
        }
        constexpr int kVAhead = NT < 2 ? NT : 2;
        bf16x8 vhs[kVAhead][2][NB], vls[kVAhead][2][NB];
        int kgo = kg;
        asm volatile("" : "+v"(kgo));       // (opaque, as in the fill: keeps the addresses inside the loop)
        auto request_values = [&](int slot, bf16x8 (&vh)[2][NB], bf16x8 (&vl)[2][NB]) __attribute__((always_inline)) {
#pragma unroll
            for (int s2 = 0; s2 < 2; ++s2) {
                const int t0 = tok0 + slot * kTileTokens + 16 * s2 + 8 * kgo;
                const int left = max(1, min(8, n - t0));
                load_values<D>(vh[s2], vl[s2], V, (size_t)g * stride + min(t0, n - 1), left, i);
            }
        };
#pragma unroll
        for (int a = 0; a < kVAhead; ++a)
            if (a < ntiles) request_values(a, vhs[a], vls[a]);
#pragma unroll
        for (int slot = 0; slot < NT; ++slot) {
            if (slot < ntiles) {
                bf16x8 vh[2][NB], vl[2][NB];
#pragma unroll
                for (int s2 = 0; s2 < 2; ++s2)
#pragma unroll
                    for (int nb = 0; nb < NB; ++nb) { vh[s2][nb] = vhs[slot % kVAhead][s2][nb]; vl[s2][nb] = vls[slot % kVAhead][s2][nb]; }
                if (slot + kVAhead < NT) {
                    if (slot + kVAhead < ntiles) request_values(slot + kVAhead, vhs[slot % kVAhead], vls[slot % kVAhead]);
                }
                f32x16 k[RB];
                res_unpack<IO, RB>(k, kq[slot]);
                float s0 = 0.f, s1 = 0.f, s2 = 0.f, s3 = 0.f;
#pragma unroll
                for (int mb = 0; mb < RB; ++mb)
#pragma unroll
                    for (int j = 0; j < 16; j += 4) {
                        s0 = fmaf(k[mb][j], vC[mb][j], s0);
                        s1 = fmaf(k[mb][j + 1], vC[mb][j + 1], s1);
                        s2 = fmaf(k[mb][j + 2], vC[mb][j + 2], s2);
                        s3 = fmaf(k[mb][j + 3], vC[mb][j + 3], s3);
                    }
                const float s = pair_sum((s0 + s1) + (s2 + s3));
                const float w = tok0 + slot * kTileTokens + i < n ? rcp_fast(s) * nm[slot] : 0.f;
#pragma unroll
                for (int mb = 0; mb < RB; ++mb)
#pragma unroll
                    for (int j = 0; j < 16; ++j) {
                        const float x = k[mb][j] * w;
                        cs[mb][j] += x;
                        const __bf16 hh = (__bf16)x;
                        const int pv = pivot_of(mb, j, kg);
                        tr_hi[pv * kTrStride + i] = __builtin_bit_cast(uint16_t, hh);
                        if (kSplit) tr_lo[pv * kTrStride + i] = __builtin_bit_cast(uint16_t, (__bf16)(x - (float)hh));
                    }
                wave_sync_lds();
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
                wave_sync_lds();
            }
            __builtin_amdgcn_sched_barrier(0);
        }
    };

    // ---- the iterations of this side.  The kept matrix is written only at the top of the outer loop (once,
    //      unless the potentials drift too far from those folded into it); the inner loop only reads it.  The
    //      last iteration is code of its own behind the loop (the keys' last sweep also contracts with V and needs
    //      registers that the loop should not have to make room for).
    auto column_sums = [&](f32x16 (&cs)[RB], int it) __attribute__((always_inline)) -> float {
        float c[16 * RB];
#pragma unroll
        for (int mb = 0; mb < RB; ++mb)
#pragma unroll
            for (int j = 0; j < 16; ++j) c[16 * mb + j] = cs[mb][j];
        float tot = reduce_scatter_tokens<16 * RB>(c, i);
        if constexpr (WS > 1) {
            // the side's wavefronts add up their shares, each in the same order: identical potentials, hence
            // identical decisions, on all of them.  One barrier per iteration on every wavefront of the
            // workgroup (both sides run p.iters iterations); the slots alternate, so that a wavefront already
            // in the next iteration does not overwrite what another one still reads.
            s_part[it & 1][wave][lane] = tot;
            __syncthreads();
            tot = 0.f;
#pragma unroll
            for (int q = 0; q < WS; ++q) tot += s_part[it & 1][side * WS + q][lane];
        }
        return fmaxf(tot * v_l, 1.0e-37f);
    };
    int it = 1;
    bool first = true, refill = true;
    do {
        fill(first);
        if (first) {
            touched<kTouchX>(touch_x);
            LOT_WSTAMP(1);
        }
        first = false;
        v_l = live ? 1.f : 0.f;
#pragma unroll
        for (int mb = 0; mb < RB; ++mb)
#pragma unroll
            for (int j = 0; j < 16; ++j) vC[mb][j] = 1.f;     // (padding pivots hold zeros in the kept matrix)
        refill = false;
        for (; it < p.iters && !refill; ++it) {
            // (the value rows are touched from inside the loop: memory operations complete in order, and whatever
            // the compiler reloads on the way into the loop would otherwise wait for these lines to arrive)
            if (it == 1 && side == 0) {
                const int last = min(n, tok0 + NT * kTileTokens);
                touch_lines<kTouchV>(touch_v, reinterpret_cast<const IO*>(p.V) + ((size_t)g * stride + min(tok0, n - 1)) * D,
                                     max(last - tok0, 0) * kRowBytes, lane);
            }
            f32x16 cs[RB];
            sweep(cs);
            const float cinv = rcp_fast(column_sums(cs, it));
            g_l += (p.eps * kLn2) * __builtin_amdgcn_logf(nbeta * cinv);
            // v for the next sweep, shifted by pivot 0's change (lane 0 holds pivot 0)
            const float d = (g_l - gref_l) * c1;
            const float d0 = __builtin_bit_cast(float, __builtin_amdgcn_readfirstlane(__builtin_bit_cast(int, d)));
            const float rel = d - d0;
            refill = __any(live && !(fabsf(rel) <= p.drift_half));   // the potentials go into the kept matrix
            v_l = live ? exp2_fast(rel) : 0.f;
            s_vec[wave][piv] = v_l;
            wave_sync_lds();
            load_pivot_vector<RB>(vC, s_vec[wave], kg);
            wave_sync_lds();
            LOT_WSTAMP(1 + min(it, 24));
        }
    } while (refill);
    {
        f32x16 cs[RB];
        if (side == 0) sweep_with_values(cs);
        else sweep(cs);
        const float cinv = rcp_fast(column_sums(cs, p.iters));
        rho_l = side == 0 ? cinv : beta_l * cinv;
        LOT_WSTAMP(1 + min(p.iters, 24));
    }

    touched<kTouchV>(touch_v);
    // ---- the two sides meet
    if (side == 0) {
        // Y'_t = v_t U_t / colsum_t: rows of this wavefront's share of U scaled per pivot, into LDS as [pivot][D]
        s_fac[part][piv] = live ? v_l * rho_l : 0.f;
        wave_sync_lds();
        f32x16 fac[RB];
        load_pivot_vector<RB>(fac, s_fac[part], kg);
#pragma unroll
        for (int mb = 0; mb < RB; ++mb)
#pragma unroll
            for (int nb = 0; nb < NB; ++nb)
#pragma unroll
                for (int j = 0; j < 16; ++j) U[mb][nb][j] *= fac[mb][j];
        if (part < kUBufs) {
#pragma unroll
            for (int mb = 0; mb < RB; ++mb)
#pragma unroll
                for (int nb = 0; nb < NB; ++nb)
#pragma unroll
                    for (int j = 0; j < 16; ++j) s_u[part][pivot_of(mb, j, kg) * D + NB * i + nb] = U[mb][nb][j];
        }
    } else if (part == 0) {
        s_qs[piv] = live ? (float)n * rho_l * v_l : 0.f;      // n rho1_t, and the v_t the expansion leaves out
    }
    if constexpr (WS > kUBufs) {
        // (a fixed order of additions: the result does not depend on which wavefront arrives first)
        __syncthreads();
        if (side == 0 && part >= kUBufs) {
#pragma unroll
            for (int mb = 0; mb < RB; ++mb)
#pragma unroll
                for (int nb = 0; nb < NB; ++nb)
#pragma unroll
                    for (int j = 0; j < 16; ++j) s_u[part - kUBufs][pivot_of(mb, j, kg) * D + NB * i + nb] += U[mb][nb][j];
        }
    }
    LOT_WSTAMP(27);
    __syncthreads();
    LOT_WSTAMP(28);

    // ---- Y''_t = n rho1_t v_t Y'_t as MFMA operand fragments (hi + lo), laid out by the whole workgroup; then the
    //      queries' wavefronts expand O = sum_t (Kt_it / s_i) Y''_t
    bf16x8* yf_hi = s_yf[0];
    bf16x8* yf_lo = s_yf[1];
    for (int f = tid; f < 2 * RB * NB * 64; f += 128 * WS) {
        const int fl = f & 63, fi = fl & 31, fkg = fl >> 5;
        const int snb = f >> 6, s = snb / NB, nb = snb % NB;
        f32x8 t;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const int pv = 32 * (s >> 1) + 16 * (s & 1) + 8 * (e >> 2) + 4 * fkg + (e & 3);
            float y = s_u[0][pv * D + NB * fi + nb];
#pragma unroll
            for (int q = 1; q < kUBufs; ++q) y += s_u[q][pv * D + NB * fi + nb];
            t[e] = y * s_qs[pv];
        }
        bf16x8 hi, lo;
        split_bf16(t, hi, lo);
        yf_hi[f] = hi;
        yf_lo[f] = lo;
    }
    __syncthreads();
    LOT_WSTAMP(29);
    if (side == 0) return;
    IO* const out = reinterpret_cast<IO*>(p.out);
#pragma unroll
    for (int slot = 0; slot < NT; ++slot) {
        if (slot < ntiles) {
            f32x16 k[RB];
            res_unpack<IO, RB>(k, kq[slot]);
            float s0 = 0.f, s1 = 0.f, s2 = 0.f, s3 = 0.f;
#pragma unroll
            for (int mb = 0; mb < RB; ++mb)
#pragma unroll
                for (int j = 0; j < 16; j += 4) {
                    s0 = fmaf(k[mb][j], vC[mb][j], s0);
                    s1 = fmaf(k[mb][j + 1], vC[mb][j + 1], s1);
                    s2 = fmaf(k[mb][j + 2], vC[mb][j + 2], s2);
                    s3 = fmaf(k[mb][j + 3], vC[mb][j + 3], s3);
                }
            const float w = rcp_fast(pair_sum((s0 + s1) + (s2 + s3)));
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
            const int row0 = tok0 + slot * kTileTokens + 4 * kg;
            IO* const lane_base = out + ((size_t)g * stride + row0) * D;
#pragma unroll
            for (int j = 0; j < 16; ++j)
                if (row0 + 8 * (j >> 2) + (j & 3) < n)
                    store_out<NB>(lane_base + (8 * (j >> 2) + (j & 3)) * D, i, oacc[0][j], oacc[NB - 1][j]);
        }
        __builtin_amdgcn_sched_barrier(0);
    }
    LOT_WSTAMP(30);
}

template <typename IO, int D, int RB, int NT, int WS, int WPE>
int launch_wave(const Args& a)
{
    const lot_shape& s = a.s;
    WaveParams p{};
    p.Q = a.Q; p.K = a.K; p.V = a.V; p.Z = a.Z; p.beta = a.beta; p.out = a.out;
    p.G = s.B * s.H; p.H = s.H; p.r = s.r; p.iters = a.iters; p.eps = a.eps;
    p.n_side[0] = a.n_k > 0 ? a.n_k : s.n;
    p.n_side[1] = a.n_q > 0 ? a.n_q : s.n;
    for (int sd = 0; sd < 2; ++sd) p.stride_side[sd] = a.n_stride > 0 ? a.n_stride : p.n_side[sd];
    p.mass_side[0] = a.mass_k; p.mass_side[1] = a.mass_q;
    p.drift_half = 0.5f * drift_limit();
#ifdef LOT_TRACE
    p.trace = (unsigned long long*)(a.ws + a.lay.fused_total);   // (developer builds: see the fused kernel)
#endif
    if (a.dry_run) {
        if (a.family_out) *a.family_out = LOT_KERNELS_KEPT_WAVEFRONT;
        return LOT_OK;
    }
    p.status = (unsigned long long*)(a.ws + a.lay.status);
    p.nonce = next_nonce();
    lot_wave_kernel<IO, D, RB, NT, WS, WPE><<<dim3((unsigned)p.G), dim3(128 * WS), 0, a.stream>>>(p);
    LOT_HIP_CHECK(hipGetLastError());
    return LOT_OK;
}

// Which variant a shape runs (NT tiles per wavefront, WS wavefronts per side, WPE wavefronts per SIMD).
//   * No more problems than compute units: every workgroup has a compute unit of its own, so a side is spread over
//     four wavefronts (eight per workgroup, two per SIMD with 256 registers each): every phase is a quarter as long,
//     for one workgroup barrier per iteration.  Up to 8, 16 or 32 tiles per side (n <= 256, 512, 1024) as far as
//     the kept words per lane stay within 64.  Measured against one or two wavefronts per side: DeiT shape
//     27 -> 21 us, B H = 192 at n = 512, r = 32 35 -> 27, B H = 8 at n = 512, r = 64 54 -> 37.
//   * Otherwise one wavefront per side with the smallest NT of {2, 4, 8} that holds the tiles (NT times the words
//     per tile at most 128), and for nine to sixteen tiles with fp32 I/O two wavefronts per side with eight tiles
//     each (bf16 I/O: four with four each, see below) -- one wavefront with sixteen would fit the registers too
//     (up to 32 pivots in bf16) but streams so many tiles one after the other, in the passes that read Q, K, V and
//     write O, that the workgroup-level kernels were faster (measured at B H = 384, n = 512: 87 us against 76).
//   * 17 to 32 tiles a side (n <= 1024, up to 32 pivots in bf16) take the form of four wavefronts with eight tiles
//     each also when the problems outnumber the compute units: the workgroups then run in rounds, which the
//     streaming kernel, the only other one such a batch has, does not make up for (B H = 264 .. 768, n = 700 and
//     1024: T = 5 76-126 us against 78-149, T = 10 90-146 against 134-245).
template <typename IO, int D, int RB>
int launch_wave_sized(const Args& a, int tiles, bool last_resort)
{
    constexpr int NW = ResWords<IO, RB>::value;
    constexpr int kMaxNT = 128 / NW;
    const bool roomy = a.s.B * a.s.H <= device_cus();
    // Where a tile takes 16 registers or more, the forms of four wavefronts per side with two wavefronts on a SIMD
    // also win when the problems outnumber the compute units: one wavefront that holds eight such tiles has the
    // SIMD to itself and nothing to hide its latencies behind (measured at B H = 264 .. 768, T = 5 and 10: bf16 I/O
    // with 64 pivots, n = 200 .. 256, 44-116 us -> 35-68; n = 400 .. 512, 98-225 us -> 71-149; fp32 I/O with 32
    // pivots level within 10 %, so that one stays as it was beyond eight tiles).  With bf16 I/O the form of four
    // wavefronts with four tiles each also takes nine to sixteen tiles of 8 words from the two wavefronts with
    // eight (same sweep, up to 32 pivots, n = 400 .. 512: T = 5 37-79 us -> 37-68, T = 10 44-90 -> 46-81; the
    // BERT shape 52 -> 49).
    constexpr bool kWide = NW >= 16;
    if (tiles <= 2) return launch_wave<IO, D, RB, 2, 1, 1>(a);
    if (roomy || (kWide && tiles > 4)) {
        if (tiles <= 8) return launch_wave<IO, D, RB, 2, 4, 2>(a);
    }
    if (roomy || !io_is_f32<IO>::value) {
        if constexpr (4 * NW <= 64) { if (tiles <= 16) return launch_wave<IO, D, RB, 4, 4, 2>(a); }
    }
    if constexpr (8 * NW <= 64) { if (tiles <= 32 && (roomy || tiles > 16)) return launch_wave<IO, D, RB, 8, 4, 2>(a); }
    // fp32 I/O with more than 32 pivots, up to 512 tokens a side: four tiles of 32 registers beside the working set
    // overflow the 256 registers of a wavefront by far, and the form lives on spilled registers.  Where the
    // workgroup-level kernels hold the problem they are faster (B H = 8 and 48: 51-76 us against 68-86); where the
    // problems are too many for those, this still beats the streaming kernel (B H = 192 .. 768: 87-270 us against
    // 143-671): so it is offered only after the workgroup-level kernels have declined.
    if constexpr (NW == 32) { if (tiles > 8 && tiles <= 16) return last_resort ? launch_wave<IO, D, RB, 4, 4, 2>(a) : LOT_ERR_PATH; }
    if constexpr (kMaxNT >= 4) { if (tiles <= 4) return launch_wave<IO, D, RB, 4, 1, 1>(a); }
    if constexpr (kMaxNT >= 8) {
        if (tiles <= 8) return launch_wave<IO, D, RB, 8, 1, 1>(a);
        if (tiles <= 16) return launch_wave<IO, D, RB, 8, 2, 1>(a);
    }
    return LOT_ERR_PATH;
}

template <typename IO>
int dispatch_wave(const Args& a, int tiles, bool last_resort)
{
    const int d = a.s.d_k, rb = a.s.r <= 32 ? 1 : 2;
    if (d == 32 && rb == 1) return launch_wave_sized<IO, 32, 1>(a, tiles, last_resort);
    if (d == 32 && rb == 2) return launch_wave_sized<IO, 32, 2>(a, tiles, last_resort);
    if (d == 64 && rb == 1) return launch_wave_sized<IO, 64, 1>(a, tiles, last_resort);
    if (d == 64 && rb == 2) return launch_wave_sized<IO, 64, 2>(a, tiles, last_resort);
    return LOT_ERR_PATH;
}

}  // namespace

// Attention where each side fits the registers of a workgroup's wavefronts; LOT_ERR_PATH otherwise.
int run_wave(const Args& a, bool last_resort)
{
    if (!fused_supports(a.s) || a.out == nullptr) return LOT_ERR_PATH;
    const int n_k = a.n_k > 0 ? a.n_k : a.s.n, n_q = a.n_q > 0 ? a.n_q : a.s.n;
    const int longer = n_k > n_q ? n_k : n_q;
    const int tiles = (longer + kTileTokens - 1) / kTileTokens;
    return a.s.io_dtype == LOT_BF16 ? dispatch_wave<uint16_t>(a, tiles, last_resort) : dispatch_wave<float>(a, tiles, last_resort);
}

}  // namespace lot
