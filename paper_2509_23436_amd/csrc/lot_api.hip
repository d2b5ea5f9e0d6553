// libLOT C ABI: argument validation, workspace carving and dispatch.  No kernels here.
#include <atomic>
#include <chrono>
#include <cmath>
#include <cstdio>
#include <cstring>

#include "lot_internal.h"

namespace lot {

hipError_t& last_hip_error()
{
    static thread_local hipError_t e = hipSuccess;
    return e;
}

unsigned long long next_nonce()
{
    // process-wide counter seeded from the clock
    static std::atomic<unsigned long long> counter{
        (unsigned long long)std::chrono::steady_clock::now().time_since_epoch().count() << 20};
    unsigned long long v = counter.fetch_add(1) + 1;
    return v ? v : counter.fetch_add(1) + 1;
}

int device_cus()
{
    static const int cus = [] {
        int dev = 0, n = 0;
        if (hipGetDevice(&dev) == hipSuccess &&
            hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && n > 0)
            return n;
        (void)hipGetLastError();   // no device: not an error of any call of ours
        return 256;
    }();
    return cus;
}

// Testing aids: process-wide knobs set through lot_debug_set (never from the environment).
static std::atomic<long long> g_knobs[LOT_KNOB_COUNT_] = {};
static std::atomic<bool> g_knob_set[LOT_KNOB_COUNT_] = {};

static bool knob(int which, long long* v)
{
    if (!g_knob_set[which].load(std::memory_order_relaxed)) return false;
    *v = g_knobs[which].load(std::memory_order_relaxed);
    return true;
}

uint32_t spin_limit()
{
    long long v;
    if (knob(LOT_KNOB_SPIN_LIMIT, &v) && v >= 0 && v <= (1ll << 30)) return (uint32_t)v;
    return 1u << 21;
}

float reshift_limit()
{
    long long v;
    int bits = 40;
    if (knob(LOT_KNOB_RESHIFT_BITS, &v) && v >= 0 && v <= 40) bits = (int)v;
    return std::ldexp(1.0f, bits);
}

bool assemble_by_iteration()
{
    long long v;
    return knob(LOT_KNOB_BWD_ASSEMBLE_BY_ITERATION, &v) && v != 0;
}

int forward_variants()
{
    long long v;
    return knob(LOT_KNOB_FWD_STREAMING, &v) && (v == 1 || v == 2) ? (int)v : 0;
}

float drift_limit()
{
    long long v;
    if (knob(LOT_KNOB_FWD_DRIFT_LIMIT, &v) && v >= 0 && v <= 32) return (float)v;
    return 32.f;
}

int grouped_one_launch_tiles()
{
    long long v;
    if (knob(LOT_KNOB_GROUPED_ONE_LAUNCH_TILES, &v) && v >= 0) return v > (1 << 20) ? (1 << 20) : (int)v;
    return 8;
}

bool sweep_keeps_similarities()
{
    long long v;
    return !(knob(LOT_KNOB_BWD_SWEEP_RECOMPUTE, &v) && v != 0);
}

bool sweep_by_launches()
{
    long long v;
    return knob(LOT_KNOB_BWD_SWEEP_LAUNCHES, &v) && v != 0;
}

static int validate_shape(const lot_shape* s)
{
    if (!s) return LOT_ERR_NULL;
    if (s->io_dtype != LOT_F32 && s->io_dtype != LOT_BF16) return LOT_ERR_DTYPE;
    if (s->B < 1 || s->H < 1 || s->n < 1 || s->d_k < 1 || s->d_v < 1 || s->r < 1) return LOT_ERR_SHAPE;
    // ranges that keep every index computation inside 63 bits and every grid inside HIP's limits
    if (s->n > (1 << 24) || s->d_k > 1024 || s->d_v > 1024 || s->r > 1024) return LOT_ERR_SHAPE;
    // (at most 2^16 problems: per-problem arrays of up to 256 x 64 elements are then indexed within 31 bits)
    if ((int64_t)s->B * s->H > (1 << 16)) return LOT_ERR_SHAPE;
    // rows of Q, K, V, out must stay 16-byte aligned for the vector loads
    const int esz = s->io_dtype == LOT_BF16 ? 2 : 4;
    if ((s->d_k * esz) % 16 != 0 || (s->d_v * esz) % 16 != 0) return LOT_ERR_SHAPE;
    return LOT_OK;
}

static bool misaligned(const void* p, size_t a) { return ((uintptr_t)p % a) != 0; }

// Which kernels a forward call runs.
enum FwdImpl { FWD_REFERENCE = 0, FWD_FUSED = 1, FWD_GROUPED = 2 };

// AUTO sends problems with fewer tokens than this on either side to the plain kernels.  The tile kernels
// form the column sums of the row-normalised kernel in the linear domain: a pivot that is far from EVERY
// token of a side (all its entries below 2^-126 of their rows' maxima) then has a sum that fp32 cannot
// hold, and its potential comes out wrong although its mass has to go somewhere.  With a handful of tokens
// and a small eps that happens (a randomised sweep found it with one or two tokens at eps = 0.02); with
// sixteen tokens it takes every one of them to lie 87 nats below its row's maximum at that pivot, which
// similarities of the workloads' scale do not produce.  The plain kernels work in the log domain
// throughout and cost nothing at this size.
constexpr int kMinFusedTokens = 16;

// s.n = the longer side (cross attention), n_short = the shorter one.  `couplings`: lot_couplings, which
// the grouped kernels do not serve.
static int pick_forward(const lot_shape& s, int n_short, int iters, int path, bool couplings, FwdImpl* impl)
{
    const bool grouped = !couplings && grouped_supports(s) && s.r > 64;
    const bool fused = fused_supports(s);
    // (astronomical iteration counts whose column sums do not fit the fused kernel's fixed-point
    // exchange format go to the plain kernels under AUTO)
    const bool fits = fused_exchange_fits(s.n, iters);
    switch (path) {
    case LOT_PATH_AUTO:
        *impl = n_short < kMinFusedTokens ? FWD_REFERENCE : grouped ? FWD_GROUPED : (fused && fits) ? FWD_FUSED : FWD_REFERENCE;
        return LOT_OK;
    case LOT_PATH_REFERENCE: *impl = FWD_REFERENCE; return LOT_OK;
    case LOT_PATH_FUSED:
        if (grouped) { *impl = FWD_GROUPED; return LOT_OK; }
        if (!fused || !fits) return LOT_ERR_PATH;
        *impl = FWD_FUSED;
        return LOT_OK;
    case LOT_PATH_STEPWISE:      // the grouped kernels take any r <= 256: launch boundaries only
        if (couplings || !grouped_supports(s)) return LOT_ERR_PATH;
        *impl = FWD_GROUPED;
        return LOT_OK;
    default: return LOT_ERR_PATH;
    }
}

// Bytes of workspace the chosen kernels use: only what they touch, so that the common case (the
// fused kernel) asks for a few megabytes and the n x r intermediates are charged to the plain path alone.
static size_t forward_need(const lot_shape& s, int iters, FwdImpl impl)
{
    switch (impl) {
    case FWD_GROUPED: return carve_grouped(s, iters).total;
    case FWD_FUSED: return carve(s).fused_total;
    default: return carve(s).total;
    }
}

static int sizing_checks(const lot_shape* shape, int iters, const size_t* bytes_out)
{
    int rc = validate_shape(shape);
    if (rc != LOT_OK) return rc;
    if (!bytes_out) return LOT_ERR_NULL;
    if (iters < 1) return LOT_ERR_ITERS;
    return LOT_OK;
}

static int common_checks(const lot_shape* s, const void* Q, const void* K, const float* Z,
                         const float* beta, float eps, int iters, void* ws)
{
    int rc = validate_shape(s);
    if (rc != LOT_OK) return rc;
    if (!Q || !K || !Z || !beta || !ws) return LOT_ERR_NULL;
    if (!(eps > 0.0f) || !std::isfinite(eps)) return LOT_ERR_EPS;
    if (iters < 1) return LOT_ERR_ITERS;
    if (misaligned(Q, 16) || misaligned(K, 16) || misaligned(Z, 4) || misaligned(beta, 4)) return LOT_ERR_ALIGN;
    if (misaligned(ws, 256)) return LOT_ERR_WORKSPACE;
    return LOT_OK;
}

}  // namespace lot

using namespace lot;

extern "C" {

int lot_workspace_bytes_path(const lot_shape* shape, int iters, int path, size_t* bytes_out)
{
    int rc = sizing_checks(shape, iters, bytes_out);
    if (rc != LOT_OK) return rc;
    FwdImpl impl;
    rc = pick_forward(*shape, shape->n, iters, path, false, &impl);
    if (rc != LOT_OK) return rc;
    size_t need = forward_need(*shape, iters, impl);
    // The [CLS] variant runs these kernels on the n - 1 other tokens with this workspace; at the one length
    // where that changes the choice of kernels the larger of the two sizes is returned.
    if (shape->n >= 2) {
        lot_shape inner = *shape;
        inner.n = shape->n - 1;
        FwdImpl inner_impl;
        if (pick_forward(inner, inner.n, iters, path, false, &inner_impl) == LOT_OK && inner_impl != impl) {
            const size_t other = forward_need(inner, iters, inner_impl);
            if (other > need) need = other;
        }
    }
    *bytes_out = need;
    return LOT_OK;
}

int lot_workspace_bytes(const lot_shape* shape, int iters, size_t* bytes_out)
{
    return lot_workspace_bytes_path(shape, iters, LOT_PATH_AUTO, bytes_out);
}

int lot_couplings_workspace_bytes(const lot_shape* shape, int iters, int path, size_t* bytes_out)
{
    int rc = sizing_checks(shape, iters, bytes_out);
    if (rc != LOT_OK) return rc;
    FwdImpl impl;
    rc = pick_forward(*shape, shape->n, iters, path, true, &impl);
    if (rc != LOT_OK) return rc;
    *bytes_out = forward_need(*shape, iters, impl);
    return LOT_OK;
}

// Shared by the dense entry point and the [CLS] variant: n_stride = tokens between consecutive
// problems in memory (0 = shape->n).
static int attention_impl(const lot_shape* shape, const void* Q, const void* K, const void* V,
                          const float* Z, const float* beta, float eps, int iters, void* out,
                          void* workspace, size_t workspace_bytes, void* hip_stream, int path, int n_stride)
{
    int rc = common_checks(shape, Q, K, Z, beta, eps, iters, workspace);
    if (rc != LOT_OK) return rc;
    if (!V || !out) return LOT_ERR_NULL;
    if (misaligned(V, 16) || misaligned(out, 16)) return LOT_ERR_ALIGN;
    FwdImpl impl;
    rc = pick_forward(*shape, shape->n, iters, path, false, &impl);
    if (rc != LOT_OK) return rc;
    if (workspace_bytes < forward_need(*shape, iters, impl)) return LOT_ERR_WORKSPACE;
    Args a{};
    a.s = *shape; a.Q = Q; a.K = K; a.V = V; a.Z = Z; a.beta = beta; a.eps = eps; a.iters = iters;
    a.out = out; a.ws = (char*)workspace; a.stream = (hipStream_t)hip_stream; a.n_stride = n_stride;
    a.stepwise = path == LOT_PATH_STEPWISE;
    if (impl == FWD_GROUPED) return run_grouped(a);   // pivot sizes beyond one register tile
    a.lay = carve(*shape);
    if (impl == FWD_FUSED) return run_fused(a, true);
    a.gamma1 = (float*)(a.ws + a.lay.gamma1);
    a.gamma2 = (float*)(a.ws + a.lay.gamma2);
    return run_reference(a, true);
}

int lot_forward_kernels(const lot_shape* shape, int iters, int path, int* kernels_out)
{
    int rc = validate_shape(shape);
    if (rc != LOT_OK) return rc;
    if (!kernels_out) return LOT_ERR_NULL;
    if (iters < 1) return LOT_ERR_ITERS;
    FwdImpl impl;
    rc = pick_forward(*shape, shape->n, iters, path, false, &impl);
    if (rc != LOT_OK) return rc;
    if (impl == FWD_REFERENCE) { *kernels_out = LOT_KERNELS_PLAIN; return LOT_OK; }
    if (impl == FWD_GROUPED) { *kernels_out = LOT_KERNELS_GROUPED; return LOT_OK; }
    // the fused path: decided exactly as a launch would be, without launching
    Args a{};
    a.s = *shape; a.eps = 1.f; a.iters = iters; a.out = (void*)shape;   // (a non-null placeholder; nothing is dereferenced)
    a.lay = carve(*shape); a.dry_run = true; a.family_out = kernels_out;
    return run_fused(a, true);
}

int lot_attention_fwd_path(const lot_shape* shape, const void* Q, const void* K, const void* V,
                           const float* Z, const float* beta, float eps, int iters, void* out,
                           void* workspace, size_t workspace_bytes, void* hip_stream, int path)
{
    return attention_impl(shape, Q, K, V, Z, beta, eps, iters, out, workspace, workspace_bytes, hip_stream, path, 0);
}

int lot_attention_cls_fwd_path(const lot_shape* shape, const void* Q, const void* K, const void* V,
                               const float* Z, const float* beta, float eps, int iters, float beta_cls,
                               void* out, void* workspace, size_t workspace_bytes, void* hip_stream, int path)
{
    int rc = validate_shape(shape);
    if (rc != LOT_OK) return rc;
    if (shape->n < 2) return LOT_ERR_SHAPE;                    // the [CLS] token and at least one other
    if (!(beta_cls > 0.0f) || !std::isfinite(beta_cls)) return LOT_ERR_EPS;
    if (!Q || !K || !V || !out) return LOT_ERR_NULL;
    // doubly-stochastic attention among tokens 1 .. n-1: the same kernels on views that skip row 0
    // (the workspace of the full shape covers the shorter one: every region grows with n)
    lot_shape inner = *shape;
    inner.n = shape->n - 1;
    const size_t esz = shape->io_dtype == LOT_BF16 ? 2 : 4;
    rc = attention_impl(&inner, (const char*)Q + shape->d_k * esz, (const char*)K + shape->d_k * esz,
                        (const char*)V + shape->d_v * esz, Z, beta, eps, iters, (char*)out + shape->d_v * esz,
                        workspace, workspace_bytes, hip_stream, path, shape->n);
    if (rc != LOT_OK) return rc;
    return run_cls_row(*shape, Q, K, V, beta_cls, out, (hipStream_t)hip_stream);
}

int lot_attention_cls_fwd(const lot_shape* shape, const void* Q, const void* K, const void* V,
                          const float* Z, const float* beta, float eps, int iters, float beta_cls,
                          void* out, void* workspace, size_t workspace_bytes, void* hip_stream)
{
    return lot_attention_cls_fwd_path(shape, Q, K, V, Z, beta, eps, iters, beta_cls, out, workspace, workspace_bytes,
                                      hip_stream, LOT_PATH_AUTO);
}

int lot_couplings_path(const lot_shape* shape, const void* Q, const void* K,
                       const float* Z, const float* beta, float eps, int iters,
                       float* gamma1, float* gamma2,
                       void* workspace, size_t workspace_bytes, void* hip_stream, int path)
{
    int rc = common_checks(shape, Q, K, Z, beta, eps, iters, workspace);
    if (rc != LOT_OK) return rc;
    if (!gamma1 || !gamma2) return LOT_ERR_NULL;
    if (misaligned(gamma1, 16) || misaligned(gamma2, 16)) return LOT_ERR_ALIGN;
    FwdImpl impl;
    rc = pick_forward(*shape, shape->n, iters, path, true, &impl);
    if (rc != LOT_OK) return rc;
    if (workspace_bytes < forward_need(*shape, iters, impl)) return LOT_ERR_WORKSPACE;
    Args a{};
    a.s = *shape; a.Q = Q; a.K = K; a.V = nullptr; a.Z = Z; a.beta = beta; a.eps = eps; a.iters = iters;
    a.out = nullptr; a.gamma1 = gamma1; a.gamma2 = gamma2;
    a.ws = (char*)workspace; a.lay = carve(*shape); a.stream = (hipStream_t)hip_stream;
    return impl == FWD_FUSED ? run_fused(a, false) : run_reference(a, false);
}

int lot_attention_fwd(const lot_shape* shape, const void* Q, const void* K, const void* V,
                      const float* Z, const float* beta, float eps, int iters, void* out,
                      void* workspace, size_t workspace_bytes, void* hip_stream)
{
    return lot_attention_fwd_path(shape, Q, K, V, Z, beta, eps, iters, out, workspace, workspace_bytes,
                                  hip_stream, LOT_PATH_AUTO);
}

int lot_couplings(const lot_shape* shape, const void* Q, const void* K,
                  const float* Z, const float* beta, float eps, int iters,
                  float* gamma1, float* gamma2,
                  void* workspace, size_t workspace_bytes, void* hip_stream)
{
    return lot_couplings_path(shape, Q, K, Z, beta, eps, iters, gamma1, gamma2, workspace, workspace_bytes,
                              hip_stream, LOT_PATH_AUTO);
}

// ---------------------------------------------------------------------------------------------
// lot_attention_fwd without a workspace argument: the scratch memory is a fixed array of this library
// ---------------------------------------------------------------------------------------------
constexpr size_t kStaticScratchBytes = (size_t)32 << 20;
constexpr int kStaticScratchDevices = 64;
// Every device that loads the library holds its own copy of this array, at its own address, until the
// process ends.  In host code the name is only a handle: the device address is asked for once per
// device (scratch_of_current_device) and that pointer is what the kernels receive.
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];
static std::atomic<void*> g_scratch_ptr[kStaticScratchDevices] = {};

static int scratch_of_current_device(void** out)
{
    int dev = -1;
    LOT_HIP_CHECK(hipGetDevice(&dev));
    if (dev < 0 || dev >= kStaticScratchDevices) {
        last_hip_error() = hipErrorInvalidDevice;
        return LOT_ERR_HIP;
    }
    void* ptr = g_scratch_ptr[dev].load(std::memory_order_acquire);
    if (ptr == nullptr) {
        // the current device's copy; two threads that race here obtain the same address
        LOT_HIP_CHECK(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));
        if (ptr == nullptr) {
            last_hip_error() = hipErrorInvalidSymbol;
            return LOT_ERR_HIP;
        }
        g_scratch_ptr[dev].store(ptr, std::memory_order_release);
    }
    *out = ptr;
    return LOT_OK;
}

size_t lot_static_scratch_bytes(void) { return kStaticScratchBytes; }

int lot_attention_fwd_static(const lot_shape* shape, const void* Q, const void* K, const void* V,
                             const float* Z, const float* beta, float eps, int iters, void* out, void* hip_stream)
{
    // everything that can be refused is refused before the first HIP call
    int rc = validate_shape(shape);
    if (rc != LOT_OK) return rc;
    if (!Q || !K || !V || !Z || !beta || !out) return LOT_ERR_NULL;
    if (!(eps > 0.0f) || !std::isfinite(eps)) return LOT_ERR_EPS;
    if (iters < 1) return LOT_ERR_ITERS;
    if (misaligned(Q, 16) || misaligned(K, 16) || misaligned(V, 16) || misaligned(out, 16) || misaligned(Z, 4) ||
        misaligned(beta, 4))
        return LOT_ERR_ALIGN;
    FwdImpl impl;
    rc = pick_forward(*shape, shape->n, iters, LOT_PATH_AUTO, false, &impl);
    if (rc != LOT_OK) return rc;
    if (forward_need(*shape, iters, impl) > kStaticScratchBytes) return LOT_ERR_SCRATCH;
    void* ws = nullptr;
    rc = scratch_of_current_device(&ws);
    if (rc != LOT_OK) return rc;
    return attention_impl(shape, Q, K, V, Z, beta, eps, iters, out, ws, kStaticScratchBytes, hip_stream, LOT_PATH_AUTO, 0);
}

static int validate_xshape(const lot_xshape* s)
{
    if (!s) return LOT_ERR_NULL;
    lot_shape q{s->B, s->H, s->n_q, s->d_k, s->d_v, s->r, s->io_dtype};
    int rc = validate_shape(&q);
    if (rc != LOT_OK) return rc;
    q.n = s->n_k;
    return validate_shape(&q);
}

// The shape the fused kernel is configured with for a cross-attention call: n = the longer side.
static lot_shape fused_view(const lot_xshape& x)
{
    return lot_shape{x.B, x.H, x.n_q > x.n_k ? x.n_q : x.n_k, x.d_k, x.d_v, x.r, x.io_dtype};
}

static size_t cross_forward_need(const lot_xshape& x, int iters, FwdImpl impl)
{
    if (impl == FWD_REFERENCE) return carve_cross(x.B, x.H, x.n_q, x.n_k, x.r, x.d_v).total;
    return forward_need(fused_view(x), iters, impl);
}

int lot_cross_workspace_bytes_path(const lot_xshape* shape, int iters, int path, size_t* bytes_out)
{
    int rc = validate_xshape(shape);
    if (rc != LOT_OK) return rc;
    if (!bytes_out) return LOT_ERR_NULL;
    if (iters < 1) return LOT_ERR_ITERS;
    FwdImpl impl;
    rc = pick_forward(fused_view(*shape), shape->n_q < shape->n_k ? shape->n_q : shape->n_k, iters, path, false, &impl);
    if (rc != LOT_OK) return rc;
    *bytes_out = cross_forward_need(*shape, iters, impl);
    return LOT_OK;
}

int lot_cross_workspace_bytes(const lot_xshape* shape, int iters, size_t* bytes_out)
{
    return lot_cross_workspace_bytes_path(shape, iters, LOT_PATH_AUTO, bytes_out);
}

int lot_cross_attention_fwd_path(const lot_xshape* shape, const void* Q, const void* K, const void* V,
                                 const float* Z, const float* beta, const float* mass_q, const float* mass_k,
                                 float eps, int iters, void* out,
                                 void* workspace, size_t workspace_bytes, void* hip_stream, int path)
{
    int rc = validate_xshape(shape);
    if (rc != LOT_OK) return rc;
    if (!Q || !K || !V || !Z || !beta || !out || !workspace) return LOT_ERR_NULL;
    if (!(eps > 0.0f) || !std::isfinite(eps)) return LOT_ERR_EPS;
    if (iters < 1) return LOT_ERR_ITERS;
    if (misaligned(Q, 16) || misaligned(K, 16) || misaligned(V, 16) || misaligned(out, 16) || misaligned(Z, 4) ||
        misaligned(beta, 4) || misaligned(mass_q, 4) || misaligned(mass_k, 4))
        return LOT_ERR_ALIGN;
    if (misaligned(workspace, 256)) return LOT_ERR_WORKSPACE;
    const lot_shape fs = fused_view(*shape);
    FwdImpl impl;
    rc = pick_forward(fs, shape->n_q < shape->n_k ? shape->n_q : shape->n_k, iters, path, false, &impl);
    if (rc != LOT_OK) return rc;
    if (workspace_bytes < cross_forward_need(*shape, iters, impl)) return LOT_ERR_WORKSPACE;
    if (impl != FWD_REFERENCE) {
        Args f{};
        f.s = fs; f.Q = Q; f.K = K; f.V = V; f.Z = Z; f.beta = beta; f.eps = eps; f.iters = iters; f.out = out;
        f.ws = (char*)workspace; f.stream = (hipStream_t)hip_stream;
        f.n_q = shape->n_q; f.n_k = shape->n_k; f.mass_q = mass_q; f.mass_k = mass_k;
        f.stepwise = path == LOT_PATH_STEPWISE;
        if (impl == FWD_GROUPED) return run_grouped(f);   // pivot sizes beyond one register tile
        f.lay = carve(fs);
        return run_fused(f, true);
    }
    CrossArgs a{};
    a.B = shape->B; a.H = shape->H; a.n_q = shape->n_q; a.n_k = shape->n_k; a.d_k = shape->d_k; a.d_v = shape->d_v;
    a.r = shape->r; a.io_dtype = shape->io_dtype;
    a.lay = carve_cross(a.B, a.H, a.n_q, a.n_k, a.r, a.d_v);
    a.Q = Q; a.K = K; a.V = V; a.Z = Z; a.beta = beta; a.mass_q = mass_q; a.mass_k = mass_k;
    a.eps = eps; a.iters = iters; a.out = out; a.ws = (char*)workspace; a.stream = (hipStream_t)hip_stream;
    return run_cross_reference(a);
}

int lot_cross_attention_fwd(const lot_xshape* shape, const void* Q, const void* K, const void* V,
                            const float* Z, const float* beta, const float* mass_q, const float* mass_k,
                            float eps, int iters, void* out,
                            void* workspace, size_t workspace_bytes, void* hip_stream)
{
    return lot_cross_attention_fwd_path(shape, Q, K, V, Z, beta, mass_q, mass_k, eps, iters, out, workspace,
                                        workspace_bytes, hip_stream, LOT_PATH_AUTO);
}

// Which kernels a backward call runs.
enum BwdImpl { BWD_PLAIN = 0, BWD_TILED = 1, BWD_GROUPED = 2 };

// AUTO sends problems of fewer tokens than this to the plain backward kernels: with so few tokens nothing
// averages out the rounding of the tiled path's bf16 (hi + lo) contractions, and gradients that vanish
// identically (a single token, say) come out as noise at 1e-3 of the other tensors' scale; the plain
// kernels are exact to fp32 rounding and cost nothing at this size.
constexpr int kMinTiledTokens = 16;
// ... and problems with at most this many pivots: the gradient of the masses is then a difference of nearly
// equal terms, which magnifies the 2^-16 of the same contractions to just above 1e-4 of its scale with fp32
// I/O, and the bf16 roundings of the tile kernels to just above 2e-2 with bf16 I/O (a randomised sweep found
// 2.02e-2 with two pivots and fifteen iterations).
constexpr int kMinTiledPivots = 2;

// s.n = the longer side; n_short = the shorter one
static int pick_backward(const lot_shape& s, int n_short, int iters, int path, BwdImpl* impl)
{
    const bool one_tile = bwd_tiled_supports(s, iters), grouped = bwd_grouped_supports(s, iters);
    const BwdImpl tile_impl = one_tile ? BWD_TILED : BWD_GROUPED;
    switch (path) {
    case LOT_PATH_AUTO: {
        bool tiled = (one_tile || grouped) && n_short >= kMinTiledTokens;
        if (s.r <= kMinTiledPivots) tiled = false;
        *impl = tiled ? tile_impl : BWD_PLAIN;
        return LOT_OK;
    }
    case LOT_PATH_REFERENCE: *impl = BWD_PLAIN; return LOT_OK;
    case LOT_PATH_FUSED:
        if (!one_tile && !grouped) return LOT_ERR_PATH;
        *impl = tile_impl;
        return LOT_OK;
    case LOT_PATH_STEPWISE:      // BWD_TILED then runs its forward sweep as one launch per pass
        if (!one_tile && !grouped) return LOT_ERR_PATH;
        *impl = tile_impl;
        return LOT_OK;
    default: return LOT_ERR_PATH;
    }
}

static size_t backward_need(const lot_shape& s, int n_q, int n_k, int iters, BwdImpl impl)
{
    switch (impl) {
    case BWD_TILED: return carve_bwd_tiled(s, iters).total;
    case BWD_GROUPED: return carve_bwd_grouped(s, iters).total;
    default: return carve_bwd_sides(s.B, s.H, n_q, n_k, s.r, s.d_k, s.d_v, iters).total;
    }
}

int lot_attention_bwd_workspace_bytes_path(const lot_shape* shape, int iters, int path, size_t* bytes_out)
{
    int rc = validate_shape(shape);
    if (rc != LOT_OK) return rc;
    if (!bytes_out) return LOT_ERR_NULL;
    if (iters < 1) return LOT_ERR_ITERS;
    if (iters > (1 << 16)) return LOT_ERR_ITERS;   // one stored vector of potentials per iteration
    BwdImpl impl;
    rc = pick_backward(*shape, shape->n, iters, path, &impl);
    if (rc != LOT_OK) return rc;
    size_t need = backward_need(*shape, shape->n, shape->n, iters, impl);
    // The [CLS] variant runs these kernels on the n - 1 other tokens with this workspace; at the one
    // length where that changes the choice of kernels the larger of the two sizes is returned.
    if (shape->n >= 2) {
        lot_shape inner = *shape;
        inner.n = shape->n - 1;
        BwdImpl inner_impl;
        if (pick_backward(inner, inner.n, iters, path, &inner_impl) == LOT_OK && inner_impl != impl) {
            const size_t other = backward_need(inner, inner.n, inner.n, iters, inner_impl);
            if (other > need) need = other;
        }
    }
    *bytes_out = need;
    return LOT_OK;
}

int lot_attention_bwd_workspace_bytes(const lot_shape* shape, int iters, size_t* bytes_out)
{
    return lot_attention_bwd_workspace_bytes_path(shape, iters, LOT_PATH_AUTO, bytes_out);
}

// n_stride: tokens between consecutive problems in the token tensors (0 = shape->n)
static int backward_impl(const lot_shape* shape, const void* Q, const void* K, const void* V,
                         const float* Z, const float* beta, float eps, int iters, const void* dO,
                         void* dQ, void* dK, void* dV, float* dZ, float* dbeta,
                         void* workspace, size_t workspace_bytes, void* hip_stream, int path, int n_stride)
{
    int rc = validate_shape(shape);
    if (rc != LOT_OK) return rc;
    if (!Q || !K || !V || !Z || !beta || !dO || !dQ || !dK || !dV || !dZ || !dbeta || !workspace) return LOT_ERR_NULL;
    if (!(eps > 0.0f) || !std::isfinite(eps)) return LOT_ERR_EPS;
    if (iters < 1 || iters > (1 << 16)) return LOT_ERR_ITERS;
    if (misaligned(Q, 16) || misaligned(K, 16) || misaligned(V, 16) || misaligned(dO, 16) || misaligned(dQ, 16) ||
        misaligned(dK, 16) || misaligned(dV, 16) || misaligned(Z, 4) || misaligned(beta, 4) || misaligned(dZ, 4) ||
        misaligned(dbeta, 4))
        return LOT_ERR_ALIGN;
    if (misaligned(workspace, 256)) return LOT_ERR_WORKSPACE;
    // the tile kernels: r <= 64 in one register tile, larger r with the pivots in groups of 64
    BwdImpl impl;
    rc = pick_backward(*shape, shape->n, iters, path, &impl);
    if (rc != LOT_OK) return rc;
    if (workspace_bytes < backward_need(*shape, shape->n, shape->n, iters, impl)) return LOT_ERR_WORKSPACE;
    BwdArgs a{};
    a.lay = carve_bwd(*shape, iters);
    a.s = *shape; a.Q = Q; a.K = K; a.V = V; a.Z = Z; a.beta = beta; a.eps = eps; a.iters = iters;
    a.dO = dO; a.dQ = dQ; a.dK = dK; a.dV = dV; a.dZ = dZ; a.dbeta = dbeta;
    a.ws = (char*)workspace; a.stream = (hipStream_t)hip_stream;
    a.n_stride = n_stride; a.stepwise = path == LOT_PATH_STEPWISE;
    if (impl == BWD_PLAIN) return run_backward(a);
    return impl == BWD_TILED ? run_backward_tiled(a) : run_backward_grouped(a);
}

int lot_attention_bwd_path(const lot_shape* shape, const void* Q, const void* K, const void* V,
                           const float* Z, const float* beta, float eps, int iters, const void* dO,
                           void* dQ, void* dK, void* dV, float* dZ, float* dbeta,
                           void* workspace, size_t workspace_bytes, void* hip_stream, int path)
{
    return backward_impl(shape, Q, K, V, Z, beta, eps, iters, dO, dQ, dK, dV, dZ, dbeta, workspace, workspace_bytes,
                         hip_stream, path, 0);
}

int lot_cross_attention_bwd_workspace_bytes_path(const lot_xshape* shape, int iters, int path, size_t* bytes_out)
{
    int rc = validate_xshape(shape);
    if (rc != LOT_OK) return rc;
    if (!bytes_out) return LOT_ERR_NULL;
    if (iters < 1 || iters > (1 << 16)) return LOT_ERR_ITERS;
    const lot_shape longer = fused_view(*shape);
    BwdImpl impl;
    rc = pick_backward(longer, shape->n_q < shape->n_k ? shape->n_q : shape->n_k, iters, path, &impl);
    if (rc != LOT_OK) return rc;
    *bytes_out = backward_need(longer, shape->n_q, shape->n_k, iters, impl);
    return LOT_OK;
}

int lot_cross_attention_bwd_workspace_bytes(const lot_xshape* shape, int iters, size_t* bytes_out)
{
    return lot_cross_attention_bwd_workspace_bytes_path(shape, iters, LOT_PATH_AUTO, bytes_out);
}

int lot_cross_attention_bwd_path(const lot_xshape* shape, const void* Q, const void* K, const void* V,
                                 const float* Z, const float* beta, const float* mass_q, const float* mass_k,
                                 float eps, int iters, const void* dO,
                                 void* dQ, void* dK, void* dV, float* dZ, float* dbeta,
                                 void* workspace, size_t workspace_bytes, void* hip_stream, int path)
{
    int rc = validate_xshape(shape);
    if (rc != LOT_OK) return rc;
    if (!Q || !K || !V || !Z || !beta || !dO || !dQ || !dK || !dV || !dZ || !dbeta || !workspace) return LOT_ERR_NULL;
    if (!(eps > 0.0f) || !std::isfinite(eps)) return LOT_ERR_EPS;
    if (iters < 1 || iters > (1 << 16)) return LOT_ERR_ITERS;
    if (misaligned(Q, 16) || misaligned(K, 16) || misaligned(V, 16) || misaligned(dO, 16) || misaligned(dQ, 16) ||
        misaligned(dK, 16) || misaligned(dV, 16) || misaligned(Z, 4) || misaligned(beta, 4) || misaligned(dZ, 4) ||
        misaligned(dbeta, 4) || misaligned(mass_q, 4) || misaligned(mass_k, 4))
        return LOT_ERR_ALIGN;
    if (misaligned(workspace, 256)) return LOT_ERR_WORKSPACE;
    const lot_shape s = fused_view(*shape);        // n = the longer side
    BwdImpl impl;
    rc = pick_backward(s, shape->n_q < shape->n_k ? shape->n_q : shape->n_k, iters, path, &impl);
    if (rc != LOT_OK) return rc;
    if (workspace_bytes < backward_need(s, shape->n_q, shape->n_k, iters, impl)) return LOT_ERR_WORKSPACE;
    BwdArgs a{};
    a.s = s; a.Q = Q; a.K = K; a.V = V; a.Z = Z; a.beta = beta; a.eps = eps; a.iters = iters;
    a.dO = dO; a.dQ = dQ; a.dK = dK; a.dV = dV; a.dZ = dZ; a.dbeta = dbeta;
    a.ws = (char*)workspace; a.stream = (hipStream_t)hip_stream;
    a.n_q = shape->n_q; a.n_k = shape->n_k; a.mass_q = mass_q; a.mass_k = mass_k;
    a.stepwise = path == LOT_PATH_STEPWISE;
    if (impl != BWD_PLAIN) return impl == BWD_TILED ? run_backward_tiled(a) : run_backward_grouped(a);
    a.lay = carve_bwd_sides(shape->B, shape->H, shape->n_q, shape->n_k, shape->r, shape->d_k, shape->d_v, iters);
    return run_backward(a);
}

int lot_cross_attention_bwd(const lot_xshape* shape, const void* Q, const void* K, const void* V,
                            const float* Z, const float* beta, const float* mass_q, const float* mass_k,
                            float eps, int iters, const void* dO,
                            void* dQ, void* dK, void* dV, float* dZ, float* dbeta,
                            void* workspace, size_t workspace_bytes, void* hip_stream)
{
    return lot_cross_attention_bwd_path(shape, Q, K, V, Z, beta, mass_q, mass_k, eps, iters, dO, dQ, dK, dV, dZ, dbeta,
                                        workspace, workspace_bytes, hip_stream, LOT_PATH_AUTO);
}

int lot_attention_cls_bwd_path(const lot_shape* shape, const void* Q, const void* K, const void* V,
                               const float* Z, const float* beta, float eps, int iters, float beta_cls, const void* dO,
                               void* dQ, void* dK, void* dV, float* dZ, float* dbeta, float* dbeta_cls,
                               void* workspace, size_t workspace_bytes, void* hip_stream, int path)
{
    int rc = validate_shape(shape);
    if (rc != LOT_OK) return rc;
    if (shape->n < 2) return LOT_ERR_SHAPE;
    if (!(beta_cls > 0.0f) || !std::isfinite(beta_cls)) return LOT_ERR_EPS;
    if (!Q || !K || !V || !dO || !dQ || !dK || !dV || !dbeta_cls) return LOT_ERR_NULL;
    if (misaligned(dbeta_cls, 4)) return LOT_ERR_ALIGN;
    // the doubly-stochastic part among tokens 1 .. n-1: the same kernels on views that skip row 0
    lot_shape inner = *shape;
    inner.n = shape->n - 1;
    const size_t esz = shape->io_dtype == LOT_BF16 ? 2 : 4;
    const size_t qk = shape->d_k * esz, vv = shape->d_v * esz;
    rc = backward_impl(&inner, (const char*)Q + qk, (const char*)K + qk, (const char*)V + vv, Z, beta, eps, iters,
                       (const char*)dO + vv, (char*)dQ + qk, (char*)dK + qk, (char*)dV + vv, dZ, dbeta,
                       workspace, workspace_bytes, hip_stream, path, shape->n);
    if (rc != LOT_OK) return rc;
    return run_cls_row_bwd(*shape, Q, K, V, dO, beta_cls, dQ, dK, dV, dbeta_cls, (hipStream_t)hip_stream);
}

int lot_attention_cls_bwd(const lot_shape* shape, const void* Q, const void* K, const void* V,
                          const float* Z, const float* beta, float eps, int iters, float beta_cls, const void* dO,
                          void* dQ, void* dK, void* dV, float* dZ, float* dbeta, float* dbeta_cls,
                          void* workspace, size_t workspace_bytes, void* hip_stream)
{
    return lot_attention_cls_bwd_path(shape, Q, K, V, Z, beta, eps, iters, beta_cls, dO, dQ, dK, dV, dZ, dbeta,
                                      dbeta_cls, workspace, workspace_bytes, hip_stream, LOT_PATH_AUTO);
}

int lot_attention_bwd(const lot_shape* shape, const void* Q, const void* K, const void* V,
                      const float* Z, const float* beta, float eps, int iters, const void* dO,
                      void* dQ, void* dK, void* dV, float* dZ, float* dbeta,
                      void* workspace, size_t workspace_bytes, void* hip_stream)
{
    return lot_attention_bwd_path(shape, Q, K, V, Z, beta, eps, iters, dO, dQ, dK, dV, dZ, dbeta, workspace,
                                  workspace_bytes, hip_stream, LOT_PATH_AUTO);
}

int lot_workspace_status(const void* workspace)
{
    if (!workspace) return LOT_ERR_NULL;
    // word 0: nonce of a launch that gave up; word 1: nonce of the last launch on this workspace
    unsigned long long words[2] = {0, 0};
    LOT_HIP_CHECK(hipDeviceSynchronize());
    LOT_HIP_CHECK(hipMemcpy(words, workspace, sizeof(words), hipMemcpyDeviceToHost));
    return lot_status_words(words);
}

int lot_workspace_status_async(const void* workspace, unsigned long long* host_words, void* hip_stream)
{
    if (!workspace || !host_words) return LOT_ERR_NULL;
    LOT_HIP_CHECK(hipMemcpyAsync(host_words, workspace, 2 * sizeof(unsigned long long), hipMemcpyDeviceToHost,
                                 (hipStream_t)hip_stream));
    return LOT_OK;
}

int lot_status_words(const unsigned long long* host_words)
{
    if (!host_words) return LOT_ERR_NULL;
    return (host_words[1] != 0 && host_words[0] == host_words[1]) ? LOT_ERR_SYNC : LOT_OK;
}

int lot_debug_set(int knob, long long value)
{
    if (knob < 0 || knob >= LOT_KNOB_COUNT_) return LOT_ERR_SHAPE;
    if (value < 0) {
        g_knob_set[knob].store(false, std::memory_order_relaxed);
        return LOT_OK;
    }
    g_knobs[knob].store(value, std::memory_order_relaxed);
    g_knob_set[knob].store(true, std::memory_order_relaxed);
    return LOT_OK;
}

const char* lot_strerror(int code)
{
    switch (code) {
    case LOT_OK: return "ok";
    case LOT_ERR_NULL: return "a required pointer is NULL";
    case LOT_ERR_SHAPE: return "a dimension is out of range or breaks row alignment";
    case LOT_ERR_EPS: return "eps must be a finite positive number";
    case LOT_ERR_ITERS: return "iters must be at least 1";
    case LOT_ERR_DTYPE: return "io_dtype is not LOT_F32 or LOT_BF16";
    case LOT_ERR_WORKSPACE: return "workspace is too small or not 256-byte aligned";
    case LOT_ERR_ALIGN: return "a tensor pointer is not sufficiently aligned";
    case LOT_ERR_HIP: return hipGetErrorString(last_hip_error());
    case LOT_ERR_PATH: return "the requested execution path does not support this shape";
    case LOT_ERR_SYNC: return "a device-side wait between workgroups gave up";
    case LOT_ERR_SCRATCH: return "the shape needs more scratch memory than the library's fixed array holds "
                                 "(use lot_attention_fwd with a workspace of the caller's)";
    default: return "unknown status";
    }
}

int lot_version(void) { return 100; }

}  // extern "C"
