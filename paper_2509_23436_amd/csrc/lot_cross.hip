// Cross attention and non-uniform token masses, plain path: queries with masses mu (n_q tokens),
// keys with masses nu (n_k tokens); padding = tokens of mass zero.  (Paper, "Empirical measures and
// pivot": mu = sum_i p1_i delta_{q_i}, nu = sum_j p2_j delta_{k_j}; "Glued coupling": the glued plan
// has marginals mu and nu; the paper names cross attention as in scope.)  The attention applied is
// the glued plan with renormalised rows, A = Diag(mu)^-1 Gamma1 Diag(beta)^-1 Gamma2, which is
// n Gamma for uniform masses.
//
// Everything is written in terms of the row log-normalisers lse_i = LSE_t((C_it + g_t)/eps) instead
// of the token potentials f_i = eps (log mass_i - lse_i): the coupling is then
// Gamma_it = mass_i exp((C_it + g_t)/eps - lse_i), a token of mass zero contributes exactly nothing
// to any sum, and row i of Diag(mu)^-1 Gamma1 is exp((C_it + g_t)/eps - lse_i) whatever its mass.
// One plain fp32 kernel per step; every reduction has a fixed order.
#include "lot_internal.h"
#include "lot_plain_kernels.h"

namespace lot {
namespace {

// Y'[g][t][c] = (1/beta_t) sum_j mass_j exp((C2_jt + g2_t)/eps - lse2_j) V_j[c]
template <typename T>
__global__ void xr_reduce_y(const float* __restrict__ C, const float* __restrict__ lse,
                            const float* __restrict__ gpot, const float* __restrict__ mass,
                            const T* __restrict__ V, const float* __restrict__ beta, float* __restrict__ Y,
                            int H, int n, int r, int dv, float eps)
{
    const int g = blockIdx.x / r, t = blockIdx.x % r;
    const float gt = gpot[g * r + t];
    for (int c = threadIdx.x; c < dv; c += blockDim.x) {
        float acc = 0.f;
        for (int j = 0; j < n; ++j) {
            const float w = mass ? mass[(size_t)g * n + j] : 1.f / (float)n;
            if (!(w > 0.f)) continue;
            const float gam = w * expf((C[((size_t)g * n + j) * r + t] + gt) / eps - lse[(size_t)g * n + j]);
            acc = fmaf(gam, ld(V, ((size_t)g * n + j) * dv + c), acc);
        }
        Y[((size_t)g * r + t) * dv + c] = acc / beta[(g % H) * r + t];
    }
}

// O[g][i][c] = sum_t exp((C1_it + g1_t)/eps - lse1_i) Y'[g][t][c]
template <typename T>
__global__ void xr_expand(const float* __restrict__ C, const float* __restrict__ lse,
                          const float* __restrict__ gpot, const float* __restrict__ Y, T* __restrict__ out,
                          size_t total, int n, int r, int dv, float eps)
{
    const size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= total) return;
    const size_t gi = idx / dv;
    const int c = (int)(idx % dv);
    const size_t g = gi / n;
    float acc = 0.f;
    for (int t = 0; t < r; ++t)
        acc = fmaf(expf((C[gi * r + t] + gpot[g * r + t]) / eps - lse[gi]), Y[(g * r + t) * dv + c], acc);
    st(out, idx, acc);
}

template <typename T>
int run_cross_reference_t(const CrossArgs& a)
{
    const int G = a.B * a.H, r = a.r;
    hipStream_t st_ = a.stream;
    const CrossWorkspace& L = a.lay;
    float* Cs[2] = {(float*)(a.ws + L.C1), (float*)(a.ws + L.C2)};
    float* lses[2] = {(float*)(a.ws + L.lse1), (float*)(a.ws + L.lse2)};
    float* gs[2] = {(float*)(a.ws + L.g1), (float*)(a.ws + L.g2)};
    float* pm = (float*)(a.ws + L.part_m);
    float* ps = (float*)(a.ws + L.part_s);
    float* Y = (float*)(a.ws + L.Y);
    const void* Xs[2] = {a.Q, a.K};
    const float* masses[2] = {a.mass_q, a.mass_k};
    const int ns[2] = {a.n_q, a.n_k};
    ref_mark<<<1, 1, 0, st_>>>((unsigned long long*)a.ws, next_nonce());
    const int width = row_group_width(r);
    for (int s = 0; s < 2; ++s) {
        const int n = ns[s], chunks = (n + kRefChunk - 1) / kRefChunk;
        const size_t total = (size_t)G * n * r, rows = (size_t)G * n;
        xr_cost<T><<<blocks_for(total, 256), 256, 0, st_>>>((const T*)Xs[s], a.Z, Cs[s], total, a.H, n, n, a.d_k, r,
                                                            a.io_dtype == LOT_BF16);
        ref_zero<<<blocks_for((size_t)G * r, 256), 256, 0, st_>>>(gs[s], (size_t)G * r);
        for (int it = 0; it < a.iters; ++it) {
            xr_row_lse<<<blocks_for(rows * width, 256), 256, 0, st_>>>(Cs[s], gs[s], lses[s], rows, n, r, a.eps, width);
            xr_col_partial<<<(unsigned)G * chunks, 64, 0, st_>>>(Cs[s], lses[s], masses[s], pm, ps, n, r, chunks, a.eps);
            xr_col_final<<<blocks_for((size_t)G * r, 256), 256, 0, st_>>>(pm, ps, a.beta, gs[s], G, a.H, r, chunks, a.eps);
        }
    }
    xr_reduce_y<T><<<(unsigned)G * r, 64, 0, st_>>>(Cs[1], lses[1], gs[1], a.mass_k, (const T*)a.V, a.beta, Y, a.H,
                                                    a.n_k, r, a.d_v, a.eps);
    const size_t total = (size_t)G * a.n_q * a.d_v;
    xr_expand<T><<<blocks_for(total, 256), 256, 0, st_>>>(Cs[0], lses[0], gs[0], Y, (T*)a.out, total, a.n_q, r, a.d_v, a.eps);
    LOT_HIP_CHECK(hipGetLastError());
    return LOT_OK;
}

}  // namespace

CrossWorkspace carve_cross(int B, int H, int n_q, int n_k, int r, int d_v)
{
    CrossWorkspace w{};
    size_t off = 256;      // the status words come first, as in the other workspaces
    auto take = [&](size_t bytes) { size_t at = off; off += (bytes + 255) / 256 * 256; return at; };
    const size_t G = (size_t)B * H;
    const size_t nmax = n_q > n_k ? n_q : n_k;
    const size_t chunks = (nmax + kRefChunk - 1) / kRefChunk;
    w.C1 = take(G * n_q * r * 4);
    w.C2 = take(G * n_k * r * 4);
    w.lse1 = take(G * n_q * 4);
    w.lse2 = take(G * n_k * 4);
    w.g1 = take(G * r * 4);
    w.g2 = take(G * r * 4);
    w.part_m = take(G * chunks * r * 4);
    w.part_s = take(G * chunks * r * 4);
    w.Y = take(G * r * d_v * 4);
    w.total = off;
    return w;
}

int run_cross_reference(const CrossArgs& a)
{
    return a.io_dtype == LOT_BF16 ? run_cross_reference_t<uint16_t>(a) : run_cross_reference_t<float>(a);
}

}  // namespace lot
