// Reference execution path of libLOT: one plain fp32 kernel per step of the method, with the
// similarity matrices, potentials and couplings materialised in the workspace.  Any shape.
// It exists for debugging, for shapes outside the fused kernel's compiled set, and as the
// route by which lot_couplings can always show every intermediate.  Every reduction has a
// fixed order, so results are reproducible bit for bit.
//
// Steps (paper, Method section): similarities C = X Z^T ("Conditional OT"); T rounds of
// token-side then pivot-side scaling in the log domain (scaling form of Gamma^(1), Gamma^(2));
// couplings; Y = Gamma2 V, Y' = Diag(beta)^-1 Y, O = n Gamma1 Y' ("Rank and complexity").
#include "lot_internal.h"
#include "lot_plain_kernels.h"

namespace lot {
namespace {

// Gamma_it = exp((C_it + f_i + g_t)/eps); side 0 -> gamma1 [g][i][t], side 1 -> gamma2 [g][t][i].
__global__ void ref_couplings(const float* __restrict__ C, const float* __restrict__ f,
                              const float* __restrict__ gpot, float* __restrict__ gamma1,
                              float* __restrict__ gamma2, int G, int n, int r, float eps)
{
    const size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const size_t per_side = (size_t)G * n * r;
    if (idx >= 2 * per_side) return;
    const int side = (int)(idx / per_side);
    size_t rem = idx % per_side;
    const size_t g = rem / ((size_t)n * r);
    rem %= (size_t)n * r;
    const size_t i = rem / r, t = rem % r;
    const size_t pair = (size_t)side * G + g;
    const float v = expf((C[idx] + f[pair * n + i] + gpot[pair * r + t]) / eps);
    if (side == 0) gamma1[(g * n + i) * r + t] = v;
    else gamma2[(g * r + t) * n + i] = v;
}

// Y'[g][t][c] = (sum_j gamma2[g][t][j] V[g][j][c]) / beta_t.  One block of 256 threads per (g, t):
// thread = (token slice s of 16, column class of 16); a thread sums every 16th token for its columns,
// the slices are then added in LDS in slice order.
constexpr int kYSlices = 16, kYCols = 16;
template <typename T>
__global__ void ref_reduce_y(const float* __restrict__ gamma2, const T* __restrict__ V,
                             const float* __restrict__ beta, float* __restrict__ Y,
                             int H, int n, int n_stride, int r, int dv)
{
    __shared__ float s_part[kYSlices][4 * kYCols];
    const int g = blockIdx.x / r, t = blockIdx.x % r;
    const int sl = threadIdx.x / kYCols, cc = threadIdx.x % kYCols;
    const float* row = gamma2 + ((size_t)g * r + t) * n;
    for (int c0 = 0; c0 < dv; c0 += 4 * kYCols) {          // four columns of a thread at a time
        float acc[4] = {0.f, 0.f, 0.f, 0.f};
        for (int j = sl; j < n; j += kYSlices) {
            const float w = row[j];
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int c = c0 + q * kYCols + cc;
                if (c < dv) acc[q] = fmaf(w, ld(V, ((size_t)g * n_stride + j) * dv + c), acc[q]);
            }
        }
#pragma unroll
        for (int q = 0; q < 4; ++q) s_part[sl][q * kYCols + cc] = acc[q];
        __syncthreads();
        if (threadIdx.x < 4 * kYCols) {
            const int c = c0 + threadIdx.x;
            float tot = 0.f;
            for (int k = 0; k < kYSlices; ++k) tot += s_part[k][threadIdx.x];
            if (c < dv) Y[((size_t)g * r + t) * dv + c] = tot / beta[(g % H) * r + t];
        }
        __syncthreads();
    }
}

// O[g][i][c] = n * sum_t gamma1[g][i][t] Y'[g][t][c]
template <typename T>
__global__ void ref_expand(const float* __restrict__ gamma1, const float* __restrict__ Y,
                           T* __restrict__ out, size_t total, int n, int n_stride, int r, int dv)
{
    const size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= total) return;
    const size_t gi = idx / dv;           // g * n + i
    const int c = (int)(idx % dv);
    const size_t g = gi / n;
    float acc = 0.f;
    for (int t = 0; t < r; ++t) acc = fmaf(gamma1[gi * r + t], Y[(g * r + t) * dv + c], acc);
    st(out, ((g * n_stride + gi % n) * dv) + c, (float)n * acc);
}


template <typename T>
int run_reference_t(const Args& a, bool want_out)
{
    const lot_shape& s = a.s;
    const int G = s.B * s.H, n = s.n, r = s.r, pairs = 2 * G;
    const int chunks = (n + kRefChunk - 1) / kRefChunk;
    float* C = (float*)(a.ws + a.lay.C);
    float* f = (float*)(a.ws + a.lay.f);
    float* g = (float*)(a.ws + a.lay.g);
    float* pm = (float*)(a.ws + a.lay.part_m);
    float* ps = (float*)(a.ws + a.lay.part_s);
    float* Y = (float*)(a.ws + a.lay.Y);
    const size_t nelem = (size_t)pairs * n * r;
    const size_t rows = (size_t)pairs * n;
    hipStream_t st_ = a.stream;
    const int nst = a.n_stride > 0 ? a.n_stride : n;
    const int width = row_group_width(r);

    ref_mark<<<1, 1, 0, st_>>>((unsigned long long*)(a.ws + a.lay.status), next_nonce());
    float* Zt = (float*)(a.ws + a.lay.Zt);
    ref_transpose_z<<<blocks_for((size_t)s.H * r * s.d_k, 256), 256, 0, st_>>>(a.Z, Zt, s.H * r * s.d_k, r, s.d_k, s.io_dtype == LOT_BF16);
    ref_cost<T><<<blocks_for(nelem, 256), 256, 0, st_>>>((const T*)a.Q, (const T*)a.K, Zt, C, G, s.H, n, nst, s.d_k, r);
    ref_zero<<<blocks_for((size_t)pairs * r, 256), 256, 0, st_>>>(g, (size_t)pairs * r);
    for (int it = 0; it < a.iters; ++it) {
        ref_f_update<<<blocks_for(rows * width, 256), 256, 0, st_>>>(C, g, f, rows, n, r, a.eps, width);
        ref_g_partial<<<(unsigned)pairs * chunks, 64, 0, st_>>>(C, f, pm, ps, n, r, chunks, a.eps);
        ref_g_final<<<blocks_for((size_t)pairs * r, 256), 256, 0, st_>>>(pm, ps, a.beta, g, pairs, G, s.H, r, chunks, a.eps);
    }
    ref_couplings<<<blocks_for(nelem, 256), 256, 0, st_>>>(C, f, g, a.gamma1, a.gamma2, G, n, r, a.eps);
    if (want_out) {
        ref_reduce_y<T><<<(unsigned)G * r, kYSlices * kYCols, 0, st_>>>(a.gamma2, (const T*)a.V, a.beta, Y, s.H, n, nst, r, s.d_v);
        const size_t total = (size_t)G * n * s.d_v;
        ref_expand<T><<<blocks_for(total, 256), 256, 0, st_>>>(a.gamma1, Y, (T*)a.out, total, n, nst, r, s.d_v);
    }
    LOT_HIP_CHECK(hipGetLastError());
    return LOT_OK;
}

// [CLS] row (paper, "[CLS] under DS attention"): a softmax row over ALL keys of the problem,
// alpha_j = softmax_j(beta_cls <q_cls, k_j>), out_cls = sum_j alpha_j v_j.  One workgroup per problem.
// The keys are taken in chunks of kClsChunk: scores of a chunk go to LDS once, the running maximum
// and normaliser are updated the usual way (rescale by exp(old max - new max)), and the chunk's
// weighted values are added; every reduction has a fixed order.
// A row product <x, row_j> is shared by kClsLanes neighbouring lanes (lane l takes columns l,
// l + kClsLanes, ...: consecutive addresses) and combined with a butterfly, which leaves the same
// sum in all of them; the keys of a chunk are dealt to these lane groups in turn.
constexpr int kClsChunk = 2048;
constexpr int kClsThreads = 1024;
constexpr int kClsLanes = 16;
constexpr int kClsGroups = kClsThreads / kClsLanes;
constexpr int kClsWaves = kClsThreads / 64;

constexpr int kClsBatch = 4;             // keys per lane group, and columns per lane, whose loads are issued together

// <x, row_j> for the keys j = first + u * step (u < kClsBatch) of one problem (rows = its [n][d]
// matrix), 0 for keys >= limit.  All loads of a batch are issued before the first product; each
// lane adds its columns in ascending order.
template <typename T>
__device__ __forceinline__ void cls_row_dots(const float* __restrict__ x, const T* __restrict__ rows, int d, int l,
                                             int first, int step, int limit, float (&out)[kClsBatch])
{
    float s[kClsBatch];
#pragma unroll
    for (int u = 0; u < kClsBatch; ++u) s[u] = 0.f;
    for (int c0 = l; c0 < d; c0 += kClsBatch * kClsLanes) {
        float v[kClsBatch][kClsBatch], xc[kClsBatch];
#pragma unroll
        for (int u = 0; u < kClsBatch; ++u)
#pragma unroll
            for (int w = 0; w < kClsBatch; ++w) {
                const int j = first + u * step, c = c0 + w * kClsLanes;
                v[u][w] = j < limit && c < d ? ld(rows, (size_t)j * d + c) : 0.f;
            }
#pragma unroll
        for (int w = 0; w < kClsBatch; ++w) xc[w] = c0 + w * kClsLanes < d ? x[c0 + w * kClsLanes] : 0.f;
#pragma unroll
        for (int u = 0; u < kClsBatch; ++u)
#pragma unroll
            for (int w = 0; w < kClsBatch; ++w) s[u] = fmaf(xc[w], v[u][w], s[u]);
    }
#pragma unroll
    for (int u = 0; u < kClsBatch; ++u) {
#pragma unroll
        for (int w = kClsLanes / 2; w > 0; w >>= 1) s[u] += __shfl_xor(s[u], w);
        out[u] = s[u];
    }
}

// maximum or sum over the workgroup, the same value in every thread: butterfly within a wave, then
// the wave results in order.  s_red holds kClsWaves floats.
template <bool kMax>
__device__ __forceinline__ float cls_reduce(float v, float* s_red)
{
#pragma unroll
    for (int w = 32; w > 0; w >>= 1) {
        const float o = __shfl_xor(v, w);
        v = kMax ? fmaxf(v, o) : v + o;
    }
    if (threadIdx.x % 64 == 0) s_red[threadIdx.x / 64] = v;
    __syncthreads();
    float r = s_red[0];
#pragma unroll
    for (int w = 1; w < kClsWaves; ++w) r = kMax ? fmaxf(r, s_red[w]) : r + s_red[w];
    __syncthreads();
    return r;
}

template <typename T>
__global__ __launch_bounds__(kClsThreads) void cls_row(const T* __restrict__ Q, const T* __restrict__ K,
                                                       const T* __restrict__ V, T* __restrict__ out, int n, int d,
                                                       int dv, float beta_cls)
{
    __shared__ float s_p[kClsChunk];
    __shared__ float s_red[kClsWaves];
    extern __shared__ float s_dyn[];        // q_cls [d], parts x dv partial sums of the output row
    float* s_q = s_dyn;
    float* s_acc = s_dyn + d;
    const size_t g = blockIdx.x;
    const int tid = threadIdx.x;
    const int grp = tid / kClsLanes, l = tid % kClsLanes;
    const int parts = kClsThreads / dv > 0 ? kClsThreads / dv : 1;      // threads per output column
    for (int c = tid; c < d; c += kClsThreads) s_q[c] = ld(Q, g * n * d + c);
    __syncthreads();
    float run_max = -INFINITY, run_z = 0.f;
    float acc = 0.f;                        // dv <= 1024: one column per thread
    for (int j0 = 0; j0 < n; j0 += kClsChunk) {
        const int cn = min(kClsChunk, n - j0);
        float m = -INFINITY;
        for (int j = grp; j < cn; j += kClsBatch * kClsGroups) {
            float sc[kClsBatch];
            cls_row_dots(s_q, K + (g * n + j0) * d, d, l, j, kClsGroups, cn, sc);
#pragma unroll
            for (int u = 0; u < kClsBatch; ++u) {
                const int ju = j + u * kClsGroups;
                if (ju < cn) {
                    if (l == 0) s_p[ju] = beta_cls * sc[u];
                    m = fmaxf(m, beta_cls * sc[u]);
                }
            }
        }
        const float new_max = fmaxf(run_max, cls_reduce<true>(m, s_red));     // also publishes s_p
        float z = 0.f;
        for (int j = tid; j < cn; j += kClsThreads) {
            const float e = expf(s_p[j] - new_max);
            s_p[j] = e;
            z += e;
        }
        z = cls_reduce<false>(z, s_red);
        const float scale = expf(run_max - new_max);      // 0 for the first chunk
        run_z = run_z * scale + z;
        run_max = new_max;
        // weighted values of the chunk: thread = (column c, part); parts interleave the keys
        const int c = tid % (kClsThreads / parts), part = tid / (kClsThreads / parts);
        float a = 0.f;
        if (c < dv && part < parts) {
#pragma unroll 4
            for (int j = part; j < cn; j += parts) a = fmaf(s_p[j], ld(V, (g * n + j0 + j) * dv + c), a);
        }
        acc = acc * scale + a;
        __syncthreads();
    }
    // combine the parts of each column in order, normalise, store
    {
        const int c = tid % (kClsThreads / parts), part = tid / (kClsThreads / parts);
        if (c < dv && part < parts) s_acc[part * dv + c] = acc;
    }
    __syncthreads();
    for (int c = tid; c < dv; c += kClsThreads) {
        float tot = 0.f;
        for (int k = 0; k < parts; ++k) tot += s_acc[k * dv + c];
        st(out, g * n * dv + c, tot / run_z);
    }
}


// Backward of the [CLS] row.  With raw_j = <q_cls, k_j>, p = softmax(beta_cls raw), out = sum_j p_j v_j
// and the incoming gradient dout:  dp_j = <dout, v_j>,  a_j = p_j (dp_j - sum_j' p_j' dp_j')  (the
// gradient with respect to beta_cls raw_j), and
//   dq_cls = beta_cls sum_j a_j k_j,   dK_j += beta_cls a_j q_cls,   dV_j += p_j dout,
//   d beta_cls = sum_j a_j raw_j.
// Rows j >= 1 of dK and dV already hold the gradient of the doubly-stochastic part and are added to;
// row 0 (the [CLS] key and value, which only this row sees) and row 0 of dQ are written.  One
// workgroup per problem, three sweeps over the keys (maximum; normaliser and sum p dp; gradients),
// the last in chunks whose a_j and p_j sit in LDS; every reduction has a fixed order.  When all keys
// fit one chunk, raw_j and dp_j are computed once, in the first sweep, and kept in LDS for the others.
template <typename T>
__global__ __launch_bounds__(kClsThreads) void cls_row_bwd(const T* __restrict__ Q, const T* __restrict__ K,
                                                           const T* __restrict__ V, const T* __restrict__ dO,
                                                           T* __restrict__ dQ, T* __restrict__ dK, T* __restrict__ dV,
                                                           float* __restrict__ dbeta_cls, int n, int d, int dv,
                                                           float beta_cls)
{
    __shared__ float s_a[kClsChunk];
    __shared__ float s_p[kClsChunk];
    __shared__ float s_raw[kClsChunk];
    __shared__ float s_dp[kClsChunk];
    __shared__ float s_red[kClsWaves];
    extern __shared__ float s_dyn[];        // q_cls [d], dout [dv], parts x d partial sums of dq_cls
    float* s_q = s_dyn;
    float* s_do = s_dyn + d;
    float* s_acc = s_dyn + d + dv;
    const size_t g = blockIdx.x;
    const int tid = threadIdx.x;
    const int grp = tid / kClsLanes, l = tid % kClsLanes;
    const bool kept = n <= kClsChunk;
    for (int c = tid; c < d; c += kClsThreads) s_q[c] = ld(Q, g * n * d + c);
    for (int c = tid; c < dv; c += kClsThreads) s_do[c] = ld(dO, g * n * dv + c);
    __syncthreads();
    // raw_j and dp_j of the keys first + u * kClsGroups (u < kClsBatch)
    auto scores = [&](int first, float (&raw)[kClsBatch]) {
        cls_row_dots(s_q, K + g * n * d, d, l, first, kClsGroups, n, raw);
    };
    auto slopes = [&](int first, float (&dp)[kClsBatch]) {
        cls_row_dots(s_do, V + g * n * dv, dv, l, first, kClsGroups, n, dp);
    };
    // sweep 1: maximum of the scaled scores
    float m = -INFINITY;
    for (int j = grp; j < n; j += kClsBatch * kClsGroups) {
        float raw[kClsBatch], dp[kClsBatch];
        scores(j, raw);
        if (kept) slopes(j, dp);
#pragma unroll
        for (int u = 0; u < kClsBatch; ++u) {
            const int ju = j + u * kClsGroups;
            if (ju < n) {
                if (kept && l == 0) { s_raw[ju] = raw[u]; s_dp[ju] = dp[u]; }
                m = fmaxf(m, beta_cls * raw[u]);
            }
        }
    }
    m = cls_reduce<true>(m, s_red);         // also publishes s_raw, s_dp
    // sweep 2: normaliser and sum_j p_j dp_j
    float z = 0.f, pd = 0.f;
    if (kept) {
        for (int j = tid; j < n; j += kClsThreads) {
            const float e = expf(beta_cls * s_raw[j] - m);
            z += e;
            pd = fmaf(e, s_dp[j], pd);
        }
    } else {
        for (int j = grp; j < n; j += kClsBatch * kClsGroups) {
            float raw[kClsBatch], dp[kClsBatch];
            scores(j, raw);
            slopes(j, dp);
#pragma unroll
            for (int u = 0; u < kClsBatch; ++u)
                if (l == 0 && j + u * kClsGroups < n) {
                    const float e = expf(beta_cls * raw[u] - m);
                    z += e;
                    pd = fmaf(e, dp[u], pd);
                }
        }
    }
    z = cls_reduce<false>(z, s_red);
    pd = cls_reduce<false>(pd, s_red) / z;
    // sweep 3, in chunks: a_j and p_j to LDS, then column-parallel updates
    const int parts = kClsThreads / d > 0 ? kClsThreads / d : 1;          // threads per column of dq_cls
    const int parts_v = kClsThreads / dv > 0 ? kClsThreads / dv : 1;
    float dq = 0.f;                         // d <= 1024: one column per thread
    float dbc = 0.f;
    for (int j0 = 0; j0 < n; j0 += kClsChunk) {
        const int cn = min(kClsChunk, n - j0);
        if (kept) {
            for (int j = tid; j < cn; j += kClsThreads) {
                const float raw = s_raw[j];
                const float pj = expf(beta_cls * raw - m) / z;
                const float a = pj * (s_dp[j] - pd);
                s_a[j] = a;
                s_p[j] = pj;
                dbc = fmaf(a, raw, dbc);
            }
        } else {
            for (int j = grp; j < cn; j += kClsBatch * kClsGroups) {
                float raw[kClsBatch], dp[kClsBatch];
                scores(j0 + j, raw);
                slopes(j0 + j, dp);
#pragma unroll
                for (int u = 0; u < kClsBatch; ++u) {
                    const int ju = j + u * kClsGroups;
                    if (l == 0 && ju < cn) {
                        const float pj = expf(beta_cls * raw[u] - m) / z;
                        const float a = pj * (dp[u] - pd);
                        s_a[ju] = a;
                        s_p[ju] = pj;
                        dbc = fmaf(a, raw[u], dbc);
                    }
                }
            }
        }
        __syncthreads();
        {
            const int c = tid % (kClsThreads / parts), part = tid / (kClsThreads / parts);
            if (c < d && part < parts) {
                float acc = 0.f;
                const float qc = beta_cls * s_q[c];
                for (int j = part; j < cn; j += kClsBatch * parts) {
                    float kv[kClsBatch], old[kClsBatch];
#pragma unroll
                    for (int u = 0; u < kClsBatch; ++u) {
                        const int ju = j + u * parts;
                        const size_t at = (g * n + j0 + ju) * d + c;
                        kv[u] = ju < cn ? ld(K, at) : 0.f;
                        old[u] = ju < cn && j0 + ju != 0 ? ld(dK, at) : 0.f;       // row 0 is written, not added to
                    }
#pragma unroll
                    for (int u = 0; u < kClsBatch; ++u) {
                        const int ju = j + u * parts;
                        if (ju < cn) {
                            acc = fmaf(s_a[ju], kv[u], acc);
                            st(dK, (g * n + j0 + ju) * d + c, old[u] + s_a[ju] * qc);
                        }
                    }
                }
                dq += acc;
            }
        }
        {
            const int c = tid % (kClsThreads / parts_v), part = tid / (kClsThreads / parts_v);
            if (c < dv && part < parts_v)
                for (int j = part; j < cn; j += kClsBatch * parts_v) {
                    float old[kClsBatch];
#pragma unroll
                    for (int u = 0; u < kClsBatch; ++u) {
                        const int ju = j + u * parts_v;
                        old[u] = ju < cn && j0 + ju != 0 ? ld(dV, (g * n + j0 + ju) * dv + c) : 0.f;
                    }
#pragma unroll
                    for (int u = 0; u < kClsBatch; ++u) {
                        const int ju = j + u * parts_v;
                        if (ju < cn) st(dV, (g * n + j0 + ju) * dv + c, old[u] + s_p[ju] * s_do[c]);
                    }
                }
        }
        __syncthreads();
    }
    // dq_cls: combine the parts of each column in order
    {
        const int c = tid % (kClsThreads / parts), part = tid / (kClsThreads / parts);
        if (c < d && part < parts) s_acc[part * d + c] = dq;
    }
    __syncthreads();
    for (int c = tid; c < d; c += kClsThreads) {
        float tot = 0.f;
        for (int k = 0; k < parts; ++k) tot += s_acc[k * d + c];
        st(dQ, g * n * d + c, beta_cls * tot);
    }
    dbc = cls_reduce<false>(dbc, s_red);
    if (tid == 0) dbeta_cls[g] = dbc;
}

}  // namespace

int run_cls_row(const lot_shape& s, const void* Q, const void* K, const void* V, float beta_cls, void* out,
                hipStream_t stream)
{
    const int G = s.B * s.H;
    const int parts = kClsThreads / s.d_v > 0 ? kClsThreads / s.d_v : 1;
    const size_t shmem = ((size_t)s.d_k + (size_t)parts * s.d_v) * sizeof(float);
    if (s.io_dtype == LOT_BF16)
        cls_row<uint16_t><<<G, kClsThreads, shmem, stream>>>((const uint16_t*)Q, (const uint16_t*)K, (const uint16_t*)V,
                                                              (uint16_t*)out, s.n, s.d_k, s.d_v, beta_cls);
    else
        cls_row<float><<<G, kClsThreads, shmem, stream>>>((const float*)Q, (const float*)K, (const float*)V,
                                                           (float*)out, s.n, s.d_k, s.d_v, beta_cls);
    LOT_HIP_CHECK(hipGetLastError());
    return LOT_OK;
}

int run_cls_row_bwd(const lot_shape& s, const void* Q, const void* K, const void* V, const void* dO, float beta_cls,
                    void* dQ, void* dK, void* dV, float* dbeta_cls, hipStream_t stream)
{
    const int G = s.B * s.H;
    const int parts = kClsThreads / s.d_k > 0 ? kClsThreads / s.d_k : 1;
    const size_t shmem = ((size_t)s.d_k + s.d_v + (size_t)parts * s.d_k) * sizeof(float);
    if (s.io_dtype == LOT_BF16)
        cls_row_bwd<uint16_t><<<G, kClsThreads, shmem, stream>>>(
            (const uint16_t*)Q, (const uint16_t*)K, (const uint16_t*)V, (const uint16_t*)dO, (uint16_t*)dQ, (uint16_t*)dK,
            (uint16_t*)dV, dbeta_cls, s.n, s.d_k, s.d_v, beta_cls);
    else
        cls_row_bwd<float><<<G, kClsThreads, shmem, stream>>>(
            (const float*)Q, (const float*)K, (const float*)V, (const float*)dO, (float*)dQ, (float*)dK, (float*)dV,
            dbeta_cls, s.n, s.d_k, s.d_v, beta_cls);
    LOT_HIP_CHECK(hipGetLastError());
    return LOT_OK;
}

int run_reference(const Args& a, bool want_out)
{
    return a.s.io_dtype == LOT_BF16 ? run_reference_t<uint16_t>(a, want_out) : run_reference_t<float>(a, want_out);
}

}  // namespace lot
