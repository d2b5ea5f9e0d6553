// Instantiations of the fused kernel that keep the kernel matrix exp(C/eps) on chip between the
// Sinkhorn iterations (queries' share in registers, keys' share in LDS; see lot_fused_kernel.h), and
// their dispatch.  A variant is taken when no wavefront would own more than NT tiles of a side.
#include "lot_fused_kernel.h"

namespace lot {
namespace {

// Largest NT per variant: what the register file (queries) and the LDS (keys) hold.  bf16 I/O keeps the
// matrix as bf16 pairs: 8 RB registers per tile; fp32 I/O as fp32: 16 RB registers per tile, and its
// pivot pieces already take up to 24 KB of LDS.
template <typename IO, int D, int RB, int WAVES, bool MASS>
int launch_resident(const Args& a)
{
    int rc = launch<IO, D, RB, WAVES, 1, MASS>(a, true);
    if (rc != LOT_ERR_PATH) return rc;
    if constexpr (!io_is_f32<IO>::value || RB == 1) {
        rc = launch<IO, D, RB, WAVES, 2, MASS>(a, true);
        if (rc != LOT_ERR_PATH) return rc;
    }
    if constexpr (!io_is_f32<IO>::value) {
        if constexpr (WAVES == 8 && D == 64 && RB == 2) {
            // Four tiles per wavefront beside the working set overflow the 256 registers a wavefront has when
            // two share a SIMD, and the spills travel to memory and back in every call.  Four wavefronts
            // per workgroup have a SIMD each, hence 512 registers: eight tiles per wavefront fit.
            rc = launch<IO, D, RB, 4, 8, MASS>(a, true);
        } else {
            rc = launch<IO, D, RB, WAVES, 4, MASS>(a, true);
        }
    }
    return rc;
}

// workgroup size as for the streaming variants (lot_fused.hip)
template <typename IO, int D, int RB>
int launch_resident_sized(const Args& a)
{
    int dev = 0, cus = 0;
    LOT_HIP_CHECK(hipGetDevice(&dev));
    LOT_HIP_CHECK(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev));
    // (token masses: instantiations of their own, so that the kernels without them stay exactly as they are)
    const bool mass = a.mass_q != nullptr || a.mass_k != nullptr;
    if constexpr (io_is_f32<IO>::value && D == 64 && RB == 2) {
        return mass ? launch_resident<IO, D, RB, 8, true>(a) : launch_resident<IO, D, RB, 8, false>(a);
    } else {
        if (a.s.B * a.s.H <= cus) return mass ? launch_resident<IO, D, RB, 8, true>(a) : launch_resident<IO, D, RB, 8, false>(a);
        return mass ? launch_resident<IO, D, RB, 4, true>(a) : launch_resident<IO, D, RB, 4, false>(a);
    }
}

template <typename IO>
int dispatch_resident(const Args& a)
{
    const int d = a.s.d_k, rb = a.s.r <= 32 ? 1 : 2;
    if (d == 32 && rb == 1) return launch_resident_sized<IO, 32, 1>(a);
    if (d == 32 && rb == 2) return launch_resident_sized<IO, 32, 2>(a);
    if (d == 64 && rb == 1) return launch_resident_sized<IO, 64, 1>(a);
    if (d == 64 && rb == 2) return launch_resident_sized<IO, 64, 2>(a);
    return LOT_ERR_PATH;
}

}  // namespace

int run_fused_resident(const Args& a)
{
    if (!fused_supports(a.s)) return LOT_ERR_PATH;
    // bf16 I/O, more than 32 pivots and few iterations: computing and storing the kernel matrix, then sweeping it once
    // more for the first column sums, costs more than the few passes it saves (measured over B H = 8 .. 16,
    // n = 4096 .. 32768: 3-15 % slower than the streaming kernel at T = 3 and 5, level or faster from T = 10).
    // Up to 32 pivots keeping it is never slower; and with fp32 I/O, where a pass of the streaming kernel is mostly
    // its similarity product (six bf16 products over pieces of every row), keeping wins from the third iteration
    // (B H = 8 .. 16, n = 1024 .. 4096, 48 and 64 pivots, T = 3, 5, 7: 45-85 us against 62-157).
    // (The testing knob that asks for these kernels overrides this.)
    if (a.s.io_dtype == LOT_BF16 && a.s.r > 32 && a.iters < 8 && forward_variants() != 2) return LOT_ERR_PATH;
    return a.s.io_dtype == LOT_BF16 ? dispatch_resident<uint16_t>(a) : dispatch_resident<float>(a);
}

}  // namespace lot
