// Internal declarations shared by the translation units of libLOT (not installed).
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "../../include/lot.h"

namespace lot {

constexpr int kTileTokens = 32;        // tokens per MFMA tile of the fused kernel
constexpr int kFusedWaves = 4;         // fewest wavefronts per workgroup of the fused kernel
constexpr int kMaxCluster = 64;        // most workgroups that share one problem
constexpr int kMaxWgsPerCu = 8;         // upper bound on co-resident workgroups per compute unit
constexpr int kRefChunk = 128;         // tokens per workgroup in the plain kernels' column reductions

inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// Compute units of the current device, asked once per process; 256 (MI355X) where no device answers,
// so that workspace sizes can still be computed on a host without a GPU.
int device_cus();
inline int max_resident_wgs() { return kMaxWgsPerCu * device_cus(); }

// Largest cluster size the fused launcher may pick for this shape (host-only arithmetic, so
// the workspace size can be computed without a device).
inline int fused_cluster_bound(const lot_shape& s)
{
    const int problems = s.B * s.H;
    const int tiles = (s.n + kTileTokens - 1) / kTileTokens;
    int c = (tiles + kFusedWaves - 1) / kFusedWaves;
    if (c > kMaxCluster) c = kMaxCluster;
    int by_capacity = max_resident_wgs() / problems;
    if (by_capacity < 1) by_capacity = 1;
    if (c > by_capacity) c = by_capacity;
    return c < 1 ? 1 : c;
}

inline bool fused_supports(const lot_shape& s)
{
    return s.d_k == s.d_v && (s.d_k == 32 || s.d_k == 64) && s.r >= 1 && s.r <= 64;
}

// Fixed-point format of the column sums that the fused kernel's workgroups exchange: a parity buffer
// receives at most iters/2 + 1 passes, each adding at most n per pivot, and must stay below 2^53 (the
// top ten bits of a word count the arrivals) with at least 8 fractional bits.  Returns the number of fractional bits, or a negative number when the
// sums do not fit (astronomical iteration counts only).
inline int fused_exchange_frac_bits(int n_longer, int iters)
{
    const double max_sum = ((double)iters / 2.0 + 1.0) * (double)n_longer;
    int bits = 0;
    while (bits < 64 && (double)(1ull << bits) < max_sum + 1.0) ++bits;   // ceil(log2(max_sum + 1))
    const int frac = 53 - bits;
    return frac >= 8 ? frac : -1;
}
inline bool fused_exchange_fits(int n_longer, int iters) { return fused_exchange_frac_bits(n_longer, iters) >= 0; }

// Carving of the caller's workspace.  All offsets are multiples of 256 bytes.
struct Workspace {
    // fused path
    size_t status;        // uint64 [0] = nonce of a launch in which a device-side wait gave up,
                          // uint64 [1] = nonce of the last launch (equal words = that launch failed)
    size_t counters;      // uint32 [G] U arrivals + uint32 [G] y-ready, zeroed per launch
    size_t counters_bytes;
    size_t cleared;       // uint64 [G]: launch nonce, written once a problem's counters are zero
    size_t colacc;        // uint64 [G][2][2][64] fixed-point column sums, zeroed per launch
    size_t colacc_bytes;
    size_t u_part;        // float [G][cluster_bound][64][d_v]
    size_t y_tile;        // float [G][64][d_v]
    size_t fused_total;   // end of the regions the fused kernel uses
    // reference path
    size_t C;             // float [2][G][n][r]
    size_t f;             // float [2][G][n]
    size_t g;             // float [2][G][r]
    size_t part_m;        // float [2][G][chunks][r]
    size_t part_s;        // float [2][G][chunks][r]
    size_t Y;             // float [G][r][d_v]
    size_t gamma1;        // float [G][n][r]   (attention via the reference path only)
    size_t gamma2;        // float [G][r][n]
    size_t Zt;            // float [H][d_k][r]: the pivots as the similarities use them, transposed
    size_t total;
};

inline Workspace carve(const lot_shape& s)
{
    Workspace w{};
    const size_t G = (size_t)s.B * s.H, n = s.n, r = s.r, dv = s.d_v;
    const size_t cb = fused_cluster_bound(s);
    const size_t chunks = (n + kRefChunk - 1) / kRefChunk;
    size_t off = 0;
    auto take = [&](size_t bytes) { size_t o = off; off = align_up(off + bytes, 256); return o; };
    w.status = take(64 * 4);
    w.counters_bytes = align_up(2 * G * 4, 256);
    w.counters = take(w.counters_bytes);
    w.cleared = take(G * 8);
    w.colacc_bytes = G * 2 * 2 * 64 * 8;
    w.colacc = take(w.colacc_bytes);
    w.u_part = take(G * cb * 64 * dv * 4);
    w.y_tile = take(G * 64 * dv * 4);
    w.fused_total = off;
    w.Zt = take((size_t)s.H * r * s.d_k * 4);
    w.C = take(2 * G * n * r * 4);
    w.f = take(2 * G * n * 4);
    w.g = take(2 * G * r * 4);
    w.part_m = take(2 * G * chunks * r * 4);
    w.part_s = take(2 * G * chunks * r * 4);
    w.Y = take(G * r * dv * 4);
    w.gamma1 = take(G * n * r * 4);
    w.gamma2 = take(G * n * r * 4);
    w.total = off;
    return w;
}

struct Args {
    lot_shape s;
    const void* Q;
    const void* K;
    const void* V;       // null for couplings
    const float* Z;
    const float* beta;
    float eps;
    int iters;
    void* out;           // null for couplings
    float* gamma1;       // null for attention on the fused path
    float* gamma2;
    char* ws;
    Workspace lay;
    hipStream_t stream;
    int n_stride;        // tokens between consecutive problems in Q, K, V, out; 0 = dense (s.n)
    // cross attention (fused path): 0 / null = as in s.n, uniform.  s.n then holds max(n_q, n_k).
    int n_q, n_k;
    const float* mass_q;
    const float* mass_k;
    bool stepwise;       // grouped kernels: one launch per step (no kernel waits for another workgroup)
    // lot_forward_kernels: decide as for a launch, launch nothing, report the family of kernels here
    bool dry_run;
    int* family_out;
};

// Workspace of the backward pass (plain path): byte offsets, multiples of 256.
struct BwdWorkspace {
    size_t C, f, ghist, part_m, part_s;   // forward recomputation: float [G (n_q + n_k)][r], row normalisers
                                          // [G (n_q + n_k)], ghist = float [iters+1][2][G][r]
    size_t gam, dgam, dC, ybuf;           // float [G (n_q + n_k)][r] each: the query side first
    size_t tx_part;                       // float [G][chunks][r][max(d_k, d_v)]
    size_t Yp, dYp, db_glue;              // float [G][r][d_v] x 2, float [G][r]
    size_t colpart, dc, rho, dg, db_pair; // float [G][chunks][r], float [2][G][r] x 4
    size_t dZ_pair, Zr;                   // float [2][G][r][d_k], float [H][r][d_k]
    size_t Zt, Yt;                        // transposed copies: float [H][d_k][r], float [G][d_v][r]
    size_t total;
};
BwdWorkspace carve_bwd(const lot_shape& s, int iters);
BwdWorkspace carve_bwd_sides(int B, int H, int n_q, int n_k, int r, int d_k, int d_v, int iters);

struct BwdArgs {
    lot_shape s;
    const void* Q;
    const void* K;
    const void* V;
    const float* Z;
    const float* beta;
    float eps;
    int iters;
    const void* dO;
    void* dQ;
    void* dK;
    void* dV;
    float* dZ;
    float* dbeta;
    int n_stride;       // tokens between consecutive problems in Q, K, V, dO, dQ, dK, dV; 0 = contiguous
    int n_q, n_k;       // tokens per problem on the query and on the key side; 0 = s.n (else s.n = the longer)
    const float* mass_q;   // [B,H,n_q] token masses, or null: uniform
    const float* mass_k;   // [B,H,n_k]
    char* ws;
    BwdWorkspace lay;
    hipStream_t stream;
    bool stepwise;         // no kernel may wait for another workgroup: the tiled sweep runs one launch per pass
};

// Workspace of the backward pass, tiled path.
struct BwdTiledWorkspace {
    size_t colacc, ghist, gram_part, gram_full, u_part, yp, dyraw, sn_part, dcs, rhop, db_pair, db_glue, dz_part, redo, cleared;
    size_t total;
    int chunks;
};
bool bwd_tiled_supports(const lot_shape& s, int iters);
BwdTiledWorkspace carve_bwd_tiled(const lot_shape& s, int iters);

// Forward with the pivots in groups of 64, one launch per step: 64 < r <= 256 under AUTO, any r <= 256 for a
// caller that asks for launch boundaries as the only synchronisation between workgroups.
struct GroupedWorkspace {
    size_t colacc, ghist, u_part, ypp, rowlse;   // status words at offset 0
    size_t total;
    int chunks;
};
bool grouped_supports(const lot_shape& s);
GroupedWorkspace carve_grouped(const lot_shape& s, int iters);
int run_grouped(const Args& a);          // attention only; LOT_ERR_PATH outside its set

// Backward for 64 < r <= 256 (pivots in groups of 64; uniform token masses).
struct BwdGroupedWorkspace {
    size_t colacc, ghist, rowlse, erow, u_part, yp, dyraw, ydv, rhop, s_part, dg_part, dcs, gmax, db_pair, db_glue, dz_part, x_part;
    size_t total;      // status words at offset 0
    int chunks;
};
bool bwd_grouped_supports(const lot_shape& s, int iters);
BwdGroupedWorkspace carve_bwd_grouped(const lot_shape& s, int iters);
int run_backward_grouped(const BwdArgs& a);   // LOT_ERR_PATH outside its set

// Cross attention / non-uniform token masses.
struct CrossWorkspace {
    size_t C1, C2, lse1, lse2, g1, g2, part_m, part_s, Y;   // plain path (status words at offset 0)
    size_t total;
};
CrossWorkspace carve_cross(int B, int H, int n_q, int n_k, int r, int d_v);
struct CrossArgs {
    int B, H, n_q, n_k, d_k, d_v, r, io_dtype;
    const void* Q;          // [B,H,n_q,d_k]
    const void* K;          // [B,H,n_k,d_k]
    const void* V;          // [B,H,n_k,d_v]
    const float* Z;
    const float* beta;
    const float* mass_q;    // [B,H,n_q] or null (uniform)
    const float* mass_k;    // [B,H,n_k] or null
    float eps;
    int iters;
    void* out;              // [B,H,n_q,d_v]
    char* ws;
    CrossWorkspace lay;
    hipStream_t stream;
};
int run_cross_reference(const CrossArgs& a);

// Each returns LOT_OK or LOT_ERR_HIP (the failing hipError_t is left in last_hip_error()).
int run_reference(const Args& a, bool want_out);
int run_fused(const Args& a, bool want_out);
// attention, each side within the registers of a workgroup's wavefronts; else LOT_ERR_PATH.  last_resort: also the forms
// that only pay where the workgroup-level kernels (run_fused_resident) have declined
int run_wave(const Args& a, bool last_resort);
int run_fused_resident(const Args& a);   // attention; LOT_ERR_PATH where the kernel matrix does not fit on chip
int run_backward(const BwdArgs& a);
int run_backward_tiled(const BwdArgs& a);
// out[b][h][0][:] = softmax_j(beta_cls <q_0, k_j>) V, j over all n tokens of the problem
int run_cls_row(const lot_shape& s, const void* Q, const void* K, const void* V, float beta_cls, void* out,
                hipStream_t stream);   // LOT_ERR_PATH when the shape is outside its set

// Adds the [CLS] row's share to dK and dV (rows >= 1; row 0 is written), writes row 0 of dQ and the
// per-problem derivative with respect to beta_cls.  Runs after the gradients of rows 1 .. n-1 are in place.
int run_cls_row_bwd(const lot_shape& s, const void* Q, const void* K, const void* V, const void* dO, float beta_cls,
                    void* dQ, void* dK, void* dV, float* dbeta_cls, hipStream_t stream);

hipError_t& last_hip_error();

// A value no earlier launch of this process has used (never zero): launches mark the workspace with
// it, so that nothing in the workspace has to be cleared by the host or by an extra kernel.
unsigned long long next_nonce();

// The backward assemble kernel normalises the rows of exponentials of all iterations of a tile with
// one shift per row instead of each iteration's exact row maximum, checks the row sums, and re-shifts
// when a sum leaves [1/limit, limit].  2^40 by default: every exponential that matters (down to 2^-24
// of the row maximum) then stays far from the ends of the fp32 range.  lot_debug_set(LOT_KNOB_RESHIFT_BITS,
// bits) with bits in 0..40 lowers the limit to 2^bits: a testing aid that makes the re-shifting branch
// run on ordinary inputs (0: practically every iteration takes it).
float reshift_limit();

// The tiled backward path assembles the similarity gradients of all iterations of a tile at once (two
// small matrix products) when there are at most 16 iterations, and redoes, iteration by iteration, only
// the workgroups in which a row sum left the range above.  lot_debug_set(LOT_KNOB_BWD_ASSEMBLE_BY_ITERATION,
// 1) sends every workgroup through the iteration-by-iteration kernel: a testing aid that keeps that
// kernel exercised on ordinary inputs.
bool assemble_by_iteration();

// Poll budget of a bounded wait between cooperating workgroups (2^21 polls by default: seconds).
// lot_debug_set(LOT_KNOB_SPIN_LIMIT, v) replaces it: a testing aid -- with 0 every wait gives up at
// once, the kernels end early and the call is reported by lot_workspace_status.
uint32_t spin_limit();

// Testing aid (LOT_KNOB_FWD_STREAMING): 1 = the fused forward never keeps the kernel matrix on chip, so that
// the variants that re-read Q and K in every pass (what long sequences run) are exercised on short ones;
// 2 = no wavefront-per-side kernel, and the workgroup-level kept-matrix variants wherever they fit (also
// where few iterations make AUTO prefer the streaming kernel), so that these are; 0 = as shipped.
int forward_variants();

// The forward kernels that keep the kernel matrix on chip recompute it when the potentials have spread
// over more than this many binary orders since it was computed (32).  Testing aid (LOT_KNOB_FWD_DRIFT_LIMIT):
// a smaller value, down to 0 (recompute in every iteration), so that this path runs on ordinary inputs.
float drift_limit();

// Testing aid (LOT_KNOB_BWD_SWEEP_LAUNCHES): run the tiled backward's forward sweep as one launch per
// pass although the persistent form would fit.
bool sweep_by_launches();
bool sweep_keeps_similarities();   // testing aid: false = the backward sweep recomputes the similarities in every pass
int grouped_one_launch_tiles();   // testing aid: tiles per workgroup up to which the grouped forward is one launch

#define LOT_HIP_CHECK(expr)                                   \
    do {                                                      \
        hipError_t e_ = (expr);                               \
        if (e_ != hipSuccess) {                               \
            ::lot::last_hip_error() = e_;                     \
            return LOT_ERR_HIP;                               \
        }                                                     \
    } while (0)

// bf16 <-> fp32 on raw bits (device and host)
__host__ __device__ inline float bf16_to_f32(uint16_t b)
{
    union { uint32_t u; float f; } v;
    v.u = (uint32_t)b << 16;
    return v.f;
}
__host__ __device__ inline uint16_t f32_to_bf16_rne(float f)
{
    union { uint32_t u; float f; } v;
    v.f = f;
    if ((v.u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((v.u >> 16) | 0x40);  // NaN stays NaN
    uint32_t bias = ((v.u >> 16) & 1u) + 0x7fffu;
    return (uint16_t)((v.u + bias) >> 16);
}

}  // namespace lot
