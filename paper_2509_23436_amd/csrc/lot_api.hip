// libLOT C ABI: argument validation, workspace carving and dispatch.  No kernels here.
#include <atomic>
#include <chrono>
#include <cmath>
#include <cstdlib>
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

uint32_t spin_limit()
{
    if (const char* e = std::getenv("LOT_SPIN_LIMIT")) {
        const long long v = std::atoll(e);
        if (v >= 0 && v <= (1ll << 30)) return (uint32_t)v;
    }
    return 1u << 21;
}

float reshift_limit()
{
    int bits = 40;
    if (const char* e = std::getenv("LOT_RESHIFT_BITS")) {
        const int v = std::atoi(e);
        if (v >= 0 && v <= 40) bits = v;
    }
    return std::ldexp(1.0f, bits);
}

bool assemble_by_iteration()
{
    const char* e = std::getenv("LOT_BWD_ASSEMBLE_BY_ITERATION");
    return e && std::atoi(e) != 0;
}

static int validate_shape(const lot_shape* s)
{
    if (!s) return LOT_ERR_NULL;
    if (s->io_dtype != LOT_F32 && s->io_dtype != LOT_BF16) return LOT_ERR_DTYPE;
    if (s->B < 1 || s->H < 1 || s->n < 1 || s->d_k < 1 || s->d_v < 1 || s->r < 1) return LOT_ERR_SHAPE;
    // ranges that keep every index computation inside 63 bits and every grid inside HIP's limits
    if (s->n > (1 << 24) || s->d_k > 1024 || s->d_v > 1024 || s->r > 1024) return LOT_ERR_SHAPE;
    if ((int64_t)s->B * s->H > (1 << 20)) return LOT_ERR_SHAPE;
    // rows of Q, K, V, out must stay 16-byte aligned for the vector loads
    const int esz = s->io_dtype == LOT_BF16 ? 2 : 4;
    if ((s->d_k * esz) % 16 != 0 || (s->d_v * esz) % 16 != 0) return LOT_ERR_SHAPE;
    return LOT_OK;
}

static bool misaligned(const void* p, size_t a) { return ((uintptr_t)p % a) != 0; }

static int common_checks(const lot_shape* s, const void* Q, const void* K, const float* Z,
                         const float* beta, float eps, int iters, void* ws, size_t ws_bytes)
{
    int rc = validate_shape(s);
    if (rc != LOT_OK) return rc;
    if (!Q || !K || !Z || !beta || !ws) return LOT_ERR_NULL;
    if (!(eps > 0.0f) || !std::isfinite(eps)) return LOT_ERR_EPS;
    if (iters < 1) return LOT_ERR_ITERS;
    if (misaligned(Q, 16) || misaligned(K, 16) || misaligned(Z, 4) || misaligned(beta, 4)) return LOT_ERR_ALIGN;
    if (misaligned(ws, 256)) return LOT_ERR_WORKSPACE;
    if (ws_bytes < carve(*s).total) return LOT_ERR_WORKSPACE;
    return LOT_OK;
}

static int pick_path(const lot_shape& s, int path, bool* fused)
{
    switch (path) {
    case LOT_PATH_AUTO: *fused = fused_supports(s); return LOT_OK;
    case LOT_PATH_REFERENCE: *fused = false; return LOT_OK;
    case LOT_PATH_FUSED:
        if (!fused_supports(s)) return LOT_ERR_PATH;
        *fused = true;
        return LOT_OK;
    default: return LOT_ERR_PATH;
    }
}

}  // namespace lot

using namespace lot;

extern "C" {

int lot_workspace_bytes(const lot_shape* shape, int iters, size_t* bytes_out)
{
    int rc = validate_shape(shape);
    if (rc != LOT_OK) return rc;
    if (!bytes_out) return LOT_ERR_NULL;
    if (iters < 1) return LOT_ERR_ITERS;
    size_t need = carve(*shape).total;
    if (grouped_supports(*shape)) {
        const size_t grouped = carve_grouped(*shape, iters).total;     // grows with iters
        if (grouped > need) need = grouped;
    }
    *bytes_out = need;
    return LOT_OK;
}

// Shared by the dense entry point and the [CLS] variant: n_stride = tokens between consecutive
// problems in memory (0 = shape->n).
static int attention_impl(const lot_shape* shape, const void* Q, const void* K, const void* V,
                          const float* Z, const float* beta, float eps, int iters, void* out,
                          void* workspace, size_t workspace_bytes, void* hip_stream, int path, int n_stride)
{
    int rc = common_checks(shape, Q, K, Z, beta, eps, iters, workspace, workspace_bytes);
    if (rc != LOT_OK) return rc;
    if (!V || !out) return LOT_ERR_NULL;
    if (misaligned(V, 16) || misaligned(out, 16)) return LOT_ERR_ALIGN;
    // pivot sizes beyond one register tile: the grouped kernels stand in for the fused one
    if (grouped_supports(*shape) && (path == LOT_PATH_AUTO || path == LOT_PATH_FUSED)) {
        if (workspace_bytes < carve_grouped(*shape, iters).total) return LOT_ERR_WORKSPACE;
        Args ga{};
        ga.s = *shape; ga.Q = Q; ga.K = K; ga.V = V; ga.Z = Z; ga.beta = beta; ga.eps = eps; ga.iters = iters;
        ga.out = out; ga.ws = (char*)workspace; ga.stream = (hipStream_t)hip_stream; ga.n_stride = n_stride;
        return run_grouped(ga);
    }
    bool fused = false;
    rc = pick_path(*shape, path, &fused);
    if (rc != LOT_OK) return rc;
    Args a{};
    a.s = *shape; a.Q = Q; a.K = K; a.V = V; a.Z = Z; a.beta = beta; a.eps = eps; a.iters = iters;
    a.out = out; a.ws = (char*)workspace; a.lay = carve(*shape); a.stream = (hipStream_t)hip_stream;
    a.n_stride = n_stride;
    if (fused) {
        rc = run_fused(a, true);
        // AUTO falls back to the reference kernels for the (astronomical) iteration counts whose
        // column sums do not fit the fused kernel's fixed-point exchange format
        if (!(rc == LOT_ERR_PATH && path == LOT_PATH_AUTO)) return rc;
    }
    a.gamma1 = (float*)(a.ws + a.lay.gamma1);
    a.gamma2 = (float*)(a.ws + a.lay.gamma2);
    return run_reference(a, true);
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
    int rc = common_checks(shape, Q, K, Z, beta, eps, iters, workspace, workspace_bytes);
    if (rc != LOT_OK) return rc;
    if (!gamma1 || !gamma2) return LOT_ERR_NULL;
    if (misaligned(gamma1, 16) || misaligned(gamma2, 16)) return LOT_ERR_ALIGN;
    bool fused = false;
    rc = pick_path(*shape, path, &fused);
    if (rc != LOT_OK) return rc;
    Args a{};
    a.s = *shape; a.Q = Q; a.K = K; a.V = nullptr; a.Z = Z; a.beta = beta; a.eps = eps; a.iters = iters;
    a.out = nullptr; a.gamma1 = gamma1; a.gamma2 = gamma2;
    a.ws = (char*)workspace; a.lay = carve(*shape); a.stream = (hipStream_t)hip_stream;
    if (fused) {
        rc = run_fused(a, false);
        if (!(rc == LOT_ERR_PATH && path == LOT_PATH_AUTO)) return rc;
    }
    return run_reference(a, false);
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

int lot_cross_workspace_bytes(const lot_xshape* shape, int iters, size_t* bytes_out)
{
    int rc = validate_xshape(shape);
    if (rc != LOT_OK) return rc;
    if (!bytes_out) return LOT_ERR_NULL;
    if (iters < 1) return LOT_ERR_ITERS;
    size_t need = carve_cross(shape->B, shape->H, shape->n_q, shape->n_k, shape->r, shape->d_v).total;
    const lot_shape fs = fused_view(*shape);
    if (fused_supports(fs)) {
        const size_t fused = carve(fs).C;      // the fused kernel's regions come first in that layout
        if (fused > need) need = fused;
    }
    if (grouped_supports(fs)) {
        const size_t grouped = carve_grouped(fs, iters).total;
        if (grouped > need) need = grouped;
    }
    *bytes_out = need;
    return LOT_OK;
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
    size_t need = 0;
    rc = lot_cross_workspace_bytes(shape, iters, &need);
    if (rc != LOT_OK) return rc;
    if (workspace_bytes < need) return LOT_ERR_WORKSPACE;
    const lot_shape fs = fused_view(*shape);
    // pivot sizes beyond one register tile: the grouped kernels stand in for the fused one
    if (grouped_supports(fs) && (path == LOT_PATH_AUTO || path == LOT_PATH_FUSED)) {
        Args ga{};
        ga.s = fs; ga.Q = Q; ga.K = K; ga.V = V; ga.Z = Z; ga.beta = beta; ga.eps = eps; ga.iters = iters; ga.out = out;
        ga.ws = (char*)workspace; ga.stream = (hipStream_t)hip_stream;
        ga.n_q = shape->n_q; ga.n_k = shape->n_k; ga.mass_q = mass_q; ga.mass_k = mass_k;
        return run_grouped(ga);
    }
    bool fused = false;
    rc = pick_path(fs, path, &fused);
    if (rc != LOT_OK) return rc;
    if (fused) {
        Args f{};
        f.s = fs; f.Q = Q; f.K = K; f.V = V; f.Z = Z; f.beta = beta; f.eps = eps; f.iters = iters; f.out = out;
        f.ws = (char*)workspace; f.lay = carve(fs); f.stream = (hipStream_t)hip_stream;
        f.n_q = shape->n_q; f.n_k = shape->n_k; f.mass_q = mass_q; f.mass_k = mass_k;
        rc = run_fused(f, true);
        if (!(rc == LOT_ERR_PATH && path == LOT_PATH_AUTO)) return rc;
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

int lot_attention_bwd_workspace_bytes(const lot_shape* shape, int iters, size_t* bytes_out)
{
    int rc = validate_shape(shape);
    if (rc != LOT_OK) return rc;
    if (!bytes_out) return LOT_ERR_NULL;
    if (iters < 1) return LOT_ERR_ITERS;
    if (iters > (1 << 16)) return LOT_ERR_ITERS;   // one stored vector of potentials per iteration
    // covers both execution paths (the plain one is the larger)
    size_t need = carve_bwd(*shape, iters).total;
    if (bwd_tiled_supports(*shape, iters)) {
        const size_t tiled = carve_bwd_tiled(*shape, iters).total;
        if (tiled > need) need = tiled;
    }
    if (bwd_grouped_supports(*shape, iters)) {
        const size_t grouped = carve_bwd_grouped(*shape, iters).total;
        if (grouped > need) need = grouped;
    }
    *bytes_out = need;
    return LOT_OK;
}

// AUTO sends problems of fewer tokens than this to the plain backward kernels: with so few tokens nothing
// averages out the rounding of the tiled path's bf16 (hi + lo) contractions, and gradients that vanish
// identically (a single token, say) come out as noise at 1e-3 of the other tensors' scale; the plain
// kernels are exact to fp32 rounding and cost nothing at this size.
constexpr int kMinTiledTokens = 16;

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
    const bool one_tile = bwd_tiled_supports(*shape, iters), grouped = bwd_grouped_supports(*shape, iters);
    bool tiled = false;
    switch (path) {
    case LOT_PATH_AUTO: tiled = (one_tile || grouped) && shape->n >= kMinTiledTokens; break;
    case LOT_PATH_REFERENCE: tiled = false; break;
    case LOT_PATH_FUSED:
        if (!one_tile && !grouped) return LOT_ERR_PATH;
        tiled = true;
        break;
    default: return LOT_ERR_PATH;
    }
    size_t need = 0;
    rc = lot_attention_bwd_workspace_bytes(shape, iters, &need);
    if (rc != LOT_OK) return rc;
    if (workspace_bytes < need) return LOT_ERR_WORKSPACE;
    BwdArgs a{};
    a.lay = carve_bwd(*shape, iters);
    a.s = *shape; a.Q = Q; a.K = K; a.V = V; a.Z = Z; a.beta = beta; a.eps = eps; a.iters = iters;
    a.dO = dO; a.dQ = dQ; a.dK = dK; a.dV = dV; a.dZ = dZ; a.dbeta = dbeta;
    a.ws = (char*)workspace; a.stream = (hipStream_t)hip_stream;
    a.n_stride = n_stride;
    if (!tiled) return run_backward(a);
    return one_tile ? run_backward_tiled(a) : run_backward_grouped(a);
}

int lot_attention_bwd_path(const lot_shape* shape, const void* Q, const void* K, const void* V,
                           const float* Z, const float* beta, float eps, int iters, const void* dO,
                           void* dQ, void* dK, void* dV, float* dZ, float* dbeta,
                           void* workspace, size_t workspace_bytes, void* hip_stream, int path)
{
    return backward_impl(shape, Q, K, V, Z, beta, eps, iters, dO, dQ, dK, dV, dZ, dbeta, workspace, workspace_bytes,
                         hip_stream, path, 0);
}

int lot_cross_attention_bwd_workspace_bytes(const lot_xshape* shape, int iters, size_t* bytes_out)
{
    int rc = validate_xshape(shape);
    if (rc != LOT_OK) return rc;
    if (!bytes_out) return LOT_ERR_NULL;
    if (iters < 1 || iters > (1 << 16)) return LOT_ERR_ITERS;
    size_t need = carve_bwd_sides(shape->B, shape->H, shape->n_q, shape->n_k, shape->r, shape->d_k, shape->d_v, iters).total;
    const lot_shape longer = fused_view(*shape);
    if (bwd_tiled_supports(longer, iters)) {
        const size_t tiled = carve_bwd_tiled(longer, iters).total;
        if (tiled > need) need = tiled;
    }
    if (bwd_grouped_supports(longer, iters)) {
        const size_t grouped = carve_bwd_grouped(longer, iters).total;
        if (grouped > need) need = grouped;
    }
    *bytes_out = need;
    return LOT_OK;
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
    size_t need = 0;
    rc = lot_cross_attention_bwd_workspace_bytes(shape, iters, &need);
    if (rc != LOT_OK) return rc;
    if (workspace_bytes < need) return LOT_ERR_WORKSPACE;
    const lot_shape s = fused_view(*shape);        // n = the longer side
    BwdArgs a{};
    a.s = s; a.Q = Q; a.K = K; a.V = V; a.Z = Z; a.beta = beta; a.eps = eps; a.iters = iters;
    a.dO = dO; a.dQ = dQ; a.dK = dK; a.dV = dV; a.dZ = dZ; a.dbeta = dbeta;
    a.ws = (char*)workspace; a.stream = (hipStream_t)hip_stream;
    a.n_q = shape->n_q; a.n_k = shape->n_k; a.mass_q = mass_q; a.mass_k = mass_k;
    const bool one_tile = bwd_tiled_supports(s, iters), grouped = bwd_grouped_supports(s, iters);
    bool tiled = false;
    switch (path) {
    case LOT_PATH_AUTO:
        tiled = (one_tile || grouped) && shape->n_q >= kMinTiledTokens && shape->n_k >= kMinTiledTokens;
        break;
    case LOT_PATH_REFERENCE: tiled = false; break;
    case LOT_PATH_FUSED:
        if (!one_tile && !grouped) return LOT_ERR_PATH;
        tiled = true;
        break;
    default: return LOT_ERR_PATH;
    }
    if (tiled) return one_tile ? run_backward_tiled(a) : run_backward_grouped(a);
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
    return (words[1] != 0 && words[0] == words[1]) ? LOT_ERR_SYNC : LOT_OK;
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
    default: return "unknown status";
    }
}

int lot_version(void) { return 100; }

}  // extern "C"
