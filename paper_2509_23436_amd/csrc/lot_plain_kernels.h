// Plain fp32 kernels shared by the reference forward path and the backward path: similarities,
// the two Sinkhorn updates in the log domain with every reduction in a fixed order, and small
// helpers.  One step of the method per kernel, nothing fused.  (Paper, Method section: similarities
// C = X Z^T; token-side then pivot-side scaling, scaling form of Gamma^(1), Gamma^(2).)
#pragma once
#include "lot_internal.h"

namespace lot {
namespace {

template <typename T> __device__ inline float ld(const T* p, size_t i);
template <> __device__ inline float ld<float>(const float* p, size_t i) { return p[i]; }
template <> __device__ inline float ld<uint16_t>(const uint16_t* p, size_t i) { return bf16_to_f32(p[i]); }

template <typename T> __device__ inline void st(T* p, size_t i, float v);
template <> __device__ inline void st<float>(float* p, size_t i, float v) { p[i] = v; }
template <> __device__ inline void st<uint16_t>(uint16_t* p, size_t i, float v) { p[i] = f32_to_bf16_rne(v); }

// Rows of the n x r arrays are walked by a group of `width` adjacent lanes (a power of two, at most 64:
// the smallest that covers min(r, 64)), so that a wavefront reads whole rows at a time; sums and maxima
// over a row are butterfly reductions over the group (a fixed order).
inline int row_group_width(int r)
{
    int w = 1;
    while (w < r && w < 64) w <<= 1;
    return w;
}
__device__ inline float group_max(float v, int width)
{
    for (int o = width >> 1; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
    return v;
}
__device__ inline float group_sum(float v, int width)
{
    for (int o = width >> 1; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}

// Zt[h][c][t] = Z[h][t][c] as the similarities use it (rounded to bf16 for bf16 I/O): transposed once, so
// that the threads of a wavefront (consecutive pivots) read consecutive addresses.
__global__ void ref_transpose_z(const float* __restrict__ Z, float* __restrict__ Zt, int count, int r, int d, int round_z)
{
    const int idx = blockIdx.x * blockDim.x + threadIdx.x;     // (h, c, t)
    if (idx >= count) return;
    const int h = idx / (r * d), c = idx / r % d, t = idx % r;
    const float z = Z[((size_t)h * r + t) * d + c];
    Zt[idx] = round_z ? bf16_to_f32(f32_to_bf16_rne(z)) : z;
}

// C[side][g][i][t] = <x_i, z_t>, x from Q (side 0) or K (side 1); Zt from ref_transpose_z.
template <typename T>
__global__ void ref_cost(const T* __restrict__ Q, const T* __restrict__ K, const float* __restrict__ Zt,
                         float* __restrict__ C, int G, int H, int n, int n_stride, int d, int r)
{
    const size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const size_t per_side = (size_t)G * n * r;
    if (idx >= 2 * per_side) return;
    const int side = (int)(idx / per_side);
    size_t rem = idx % per_side;
    const int g = (int)(rem / ((size_t)n * r));
    rem %= (size_t)n * r;
    const int i = (int)(rem / r), t = (int)(rem % r);
    const T* x = (side == 0 ? Q : K) + ((size_t)g * n_stride + i) * d;
    const float* z = Zt + (size_t)(g % H) * d * r + t;
    float acc = 0.f;
    for (int c = 0; c < d; ++c) acc = fmaf(ld(x, c), z[(size_t)c * r], acc);
    C[idx] = acc;
}

// Marks the workspace as used by a launch that cannot fail on the device: word 1 of the status area
// takes a fresh nonce, which word 0 (written only by a launch that gave up) cannot hold.
__global__ void ref_mark(unsigned long long* status, unsigned long long nonce) { status[1] = nonce; }

__global__ void ref_zero(float* p, size_t count)
{
    const size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx < count) p[idx] = 0.f;
}

// f_i = eps (log(1/n) - LSE_t((C_it + g_t)/eps)), `width` lanes per (side, g, i).
__global__ void ref_f_update(const float* __restrict__ C, const float* __restrict__ gpot,
                             float* __restrict__ f, size_t rows, int n, int r, float eps, int width)
{
    const size_t tid = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const size_t row = min(tid / width, rows - 1);          // lanes past the end repeat the last row, store nothing
    const int sub = (int)(tid % width);
    const float* c = C + row * r;
    const float* g = gpot + (row / n) * r;
    float m = -INFINITY;
    for (int t = sub; t < r; t += width) m = fmaxf(m, (c[t] + g[t]) / eps);
    m = group_max(m, width);
    float s = 0.f;
    for (int t = sub; t < r; t += width) s += expf((c[t] + g[t]) / eps - m);
    s = group_sum(s, width);
    if (sub == 0 && tid / width < rows) f[row] = eps * (-logf((float)n) - (m + logf(s)));
}

// Per (pair, chunk of tokens, pivot): running maximum and scaled sum of exp((C_it + f_i)/eps).
__global__ void ref_g_partial(const float* __restrict__ C, const float* __restrict__ f,
                              float* __restrict__ part_m, float* __restrict__ part_s,
                              int n, int r, int chunks, float eps)
{
    const int pair = blockIdx.x / chunks, chunk = blockIdx.x % chunks;
    const int i0 = chunk * kRefChunk;
    const int i1 = min(n, i0 + kRefChunk);
    for (int t = threadIdx.x; t < r; t += blockDim.x) {
        float m = -INFINITY, s = 0.f;
        for (int i = i0; i < i1; ++i) {
            const float x = (C[((size_t)pair * n + i) * r + t] + f[(size_t)pair * n + i]) / eps;
            if (x > m) { s = s * expf(m - x) + 1.f; m = x; }
            else s += expf(x - m);
        }
        part_m[((size_t)pair * chunks + chunk) * r + t] = m;
        part_s[((size_t)pair * chunks + chunk) * r + t] = s;
    }
}

// g_t = eps (log beta_t - LSE over all tokens), combining the chunks in index order.
__global__ void ref_g_final(const float* __restrict__ part_m, const float* __restrict__ part_s,
                            const float* __restrict__ beta, float* __restrict__ gpot,
                            int pairs, int G, int H, int r, int chunks, float eps)
{
    const int idx = blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= pairs * r) return;
    const int pair = idx / r, t = idx % r;
    const int h = (pair % G) % H;
    float m = -INFINITY;
    for (int k = 0; k < chunks; ++k) m = fmaxf(m, part_m[((size_t)pair * chunks + k) * r + t]);
    float s = 0.f;
    for (int k = 0; k < chunks; ++k)
        s += part_s[((size_t)pair * chunks + k) * r + t] * expf(part_m[((size_t)pair * chunks + k) * r + t] - m);
    gpot[idx] = eps * (logf(beta[h * r + t]) - (m + logf(s)));
}

// Kernels of one Sinkhorn solve with token masses, written in terms of the row log-normalisers
// lse_i = LSE_t((C_it + g_t)/eps) (a token of mass zero then contributes exactly nothing).
// C[g][i][t] = <x_i, z_t> for one side (n tokens per problem, n_stride rows between problems)
template <typename T>
__global__ void xr_cost(const T* __restrict__ X, const float* __restrict__ Z, float* __restrict__ C,
                        size_t total, int H, int n, int n_stride, int d, int r, int round_z)
{
    const size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= total) return;
    const size_t gi = idx / r;
    const int t = (int)(idx % r);
    const int g = (int)(gi / n);
    const T* x = X + ((size_t)g * n_stride + gi % n) * d;
    const float* z = Z + ((size_t)(g % H) * r + t) * d;
    float acc = 0.f;
    for (int c = 0; c < d; ++c) {
        float zv = z[c];
        if (round_z) zv = bf16_to_f32(f32_to_bf16_rne(zv));
        acc = fmaf(ld(x, c), zv, acc);
    }
    C[idx] = acc;
}

// lse_i = LSE_t((C_it + g_t)/eps), `width` lanes per (g, i)
__global__ void xr_row_lse(const float* __restrict__ C, const float* __restrict__ gpot, float* __restrict__ lse,
                           size_t rows, int n, int r, float eps, int width)
{
    const size_t tid = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const size_t row = min(tid / width, rows - 1);          // lanes past the end repeat the last row, store nothing
    const int sub = (int)(tid % width);
    const float* c = C + row * r;
    const float* g = gpot + (row / n) * r;
    float m = -INFINITY;
    for (int t = sub; t < r; t += width) m = fmaxf(m, (c[t] + g[t]) / eps);
    m = group_max(m, width);
    float s = 0.f;
    for (int t = sub; t < r; t += width) s += expf((c[t] + g[t]) / eps - m);
    s = group_sum(s, width);
    if (sub == 0 && tid / width < rows) lse[row] = m + logf(s);
}

// per (g, chunk, t): running maximum and scaled sum of mass_i exp(C_it/eps - lse_i) over the chunk
__global__ void xr_col_partial(const float* __restrict__ C, const float* __restrict__ lse,
                               const float* __restrict__ mass, float* __restrict__ part_m,
                               float* __restrict__ part_s, int n, int r, int chunks, float eps)
{
    const int g = blockIdx.x / chunks, chunk = blockIdx.x % chunks;
    const int i0 = chunk * kRefChunk, i1 = min(n, i0 + kRefChunk);
    for (int t = threadIdx.x; t < r; t += blockDim.x) {
        float m = -INFINITY, s = 0.f;
        for (int i = i0; i < i1; ++i) {
            const float w = mass ? mass[(size_t)g * n + i] : 1.f / (float)n;
            if (!(w > 0.f)) continue;
            const float x = C[((size_t)g * n + i) * r + t] / eps - lse[(size_t)g * n + i] + logf(w);
            if (x > m) { s = s * expf(m - x) + 1.f; m = x; }
            else s += expf(x - m);
        }
        part_m[((size_t)g * chunks + chunk) * r + t] = m;
        part_s[((size_t)g * chunks + chunk) * r + t] = s;
    }
}

// g_t = eps (log beta_t - LSE_i(C_it/eps - lse_i + log mass_i)), chunks combined in index order
__global__ void xr_col_final(const float* __restrict__ part_m, const float* __restrict__ part_s,
                             const float* __restrict__ beta, float* __restrict__ gpot, int G, int H, int r,
                             int chunks, float eps)
{
    const int idx = blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= G * r) return;
    const int g = idx / r, t = idx % r;
    float m = -INFINITY;
    for (int k = 0; k < chunks; ++k) m = fmaxf(m, part_m[((size_t)g * chunks + k) * r + t]);
    float s = 0.f;
    for (int k = 0; k < chunks; ++k) {
        const float pm = part_m[((size_t)g * chunks + k) * r + t];
        if (pm > -INFINITY) s += part_s[((size_t)g * chunks + k) * r + t] * expf(pm - m);
    }
    gpot[idx] = eps * (logf(beta[(g % H) * r + t]) - (m + logf(s)));
}

inline unsigned blocks_for(size_t count, int threads) { return (unsigned)((count + threads - 1) / threads); }

}  // namespace
}  // namespace lot
