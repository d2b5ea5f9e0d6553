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
#include "lot_fused_kernel.h"

namespace lot {
namespace {

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
        return launch<IO, D, RB, 8, 0>(a, want_out);
    } else {
        if (a.s.B * a.s.H <= cus) return launch<IO, D, RB, 8, 0>(a, want_out);
        return launch<IO, D, RB, 4, 0>(a, want_out);
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
    // the variants that keep the kernel matrix on chip, where a workgroup's share of it fits
    if (want_out && forward_variants() != 1) {
        // short sequences: a workgroup per problem, the whole kernel matrix in its wavefronts' registers
        if (forward_variants() != 2) {
            const int rc = run_wave(a, false);
            if (rc != LOT_ERR_PATH) return rc;
        }
        const int rc = run_fused_resident(a);
        if (rc != LOT_ERR_PATH) return rc;
        if (forward_variants() != 2) {
            const int rc_wave = run_wave(a, true);
            if (rc_wave != LOT_ERR_PATH) return rc_wave;
        }
    }
    return a.s.io_dtype == LOT_BF16 ? dispatch<uint16_t>(a, want_out) : dispatch<float>(a, want_out);
}

}  // namespace lot
