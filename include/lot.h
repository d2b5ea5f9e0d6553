/*
 * libLOT -- LOT attention, forward and backward, on AMD MI355X (gfx950): C ABI.
 *
 * The operation (paper, Method section, "Conditional OT", "Glued coupling and
 * doubly-stochastic attention", eq. (lotattn), "Rank and complexity"): for every (batch, head)
 * problem, with queries Q and keys K (n tokens each, uniform masses 1/n) and a per-head pivot
 * measure with r locations Z and masses beta,
 *
 *     C1 = Q Z^T,  C2 = K Z^T                                   (n x r similarities)
 *     Gamma1 = T Sinkhorn iterations on exp(C1/eps), marginals (1/n, beta)     n x r
 *     Gamma2 = transpose of the same for C2                                    r x n
 *     O = n * Gamma1 * Diag(beta)^-1 * (Gamma2 * V)                            n x d_v
 *
 * One Sinkhorn iteration is a token-side scaling followed by a pivot-side scaling, started from
 * the pivot-side scaling vector equal to one; there is no convergence test.  The n x n matrix
 * n * Gamma1 Diag(beta)^-1 Gamma2 is never formed.
 *
 * Conventions for every entry point
 *  - All tensor pointers are DEVICE pointers owned by the caller; the library allocates and frees
 *    nothing and keeps no state between calls that a result depends on (a launch counter and cached
 *    device properties only).  Outputs must not alias inputs or the workspace.
 *  - Layout: dense row-major, last index fastest.
 *        Q, K : [B, H, n, d_k]      V, out : [B, H, n, d_v]      (element type = shape.io_dtype)
 *        Z    : [H, r, d_k] float   beta   : [H, r] float        (one pivot measure per head)
 *        gamma1 : [B, H, n, r] float    gamma2 : [B, H, r, n] float
 *    Q, K, V, out must be 16-byte aligned; workspace 256-byte aligned.
 *  - beta must be strictly positive and sum to one per head (the paper's p^0); this is a caller
 *    precondition and is not checked.
 *  - With io_dtype = LOT_BF16 the similarities are computed from bf16 operands with fp32
 *    accumulation: Z (fp32, e.g. a learnable parameter) is rounded to bf16 (nearest even) inside
 *    the library, like the Q and K it meets.  The bf16 tolerance (2e-2 of the largest output) is
 *    quoted for any fp32 Z, not only for bf16-representable ones.  With LOT_F32 they are
 *    accurate to fp32 rounding (fp32 matrix instructions, or bf16 products over exact three-way
 *    pieces of the operands).  Potentials, sums and the r x d_v intermediate are fp32 in both
 *    modes.  The output is rounded to io_dtype.
 *  - Work is enqueued on `hip_stream` (a hipStream_t passed as void*, NULL = default stream) and
 *    the call returns without synchronising.  Results are bit-identical from run to run.
 *  - Return value: LOT_OK (0) or a negative lot_status.  Argument validation happens before any
 *    HIP call.  No exception or abort crosses this boundary.
 */
#ifndef LOT_H
#define LOT_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum { LOT_F32 = 0, LOT_BF16 = 1 } lot_dtype;

typedef enum {
    LOT_OK = 0,
    LOT_ERR_NULL = -1,       /* a required pointer is NULL */
    LOT_ERR_SHAPE = -2,      /* a dimension is < 1 or beyond the supported range */
    LOT_ERR_EPS = -3,        /* eps is not a finite positive number */
    LOT_ERR_ITERS = -4,      /* iters < 1 */
    LOT_ERR_DTYPE = -5,      /* io_dtype is not a lot_dtype */
    LOT_ERR_WORKSPACE = -6,  /* workspace too small or misaligned */
    LOT_ERR_ALIGN = -7,      /* a tensor pointer is not 16-byte aligned */
    LOT_ERR_HIP = -8,        /* a HIP call failed (see lot_strerror) */
    LOT_ERR_PATH = -9,       /* the requested execution path does not support this shape */
    LOT_ERR_SYNC = -10,      /* lot_workspace_status / lot_status_words: a device-side wait gave up */
    LOT_ERR_SCRATCH = -11    /* lot_attention_fwd_static: the shape needs more than the fixed scratch array */
} lot_status;

typedef struct {
    int32_t B, H;        /* batch, heads */
    int32_t n;           /* tokens (queries = keys) */
    int32_t d_k, d_v;    /* head dims of Q/K and of V/out */
    int32_t r;           /* pivot size */
    int32_t io_dtype;    /* lot_dtype of Q, K, V, out */
} lot_shape;

/* Which kernels run.  AUTO picks FUSED when the shape is in its compiled set and both sides have at least
 * 16 tokens, else REFERENCE (with a handful of tokens and a small eps a pivot can be so far from every
 * token of a side that its column sum leaves the fp32 range in the tile kernels' linear-domain sums; the
 * plain kernels work in the log domain throughout). */
typedef enum {
    LOT_PATH_AUTO = 0,
    LOT_PATH_REFERENCE = 1,  /* one plain kernel per step, similarities materialised (any shape) */
    LOT_PATH_FUSED = 2,      /* MFMA kernels; d_k = d_v in {32, 64}: r <= 64 one kernel per call (see
                                lot_forward_kernels for its families), 64 < r <= 256 grouped kernels
                                (attention only) */
    LOT_PATH_STEPWISE = 3    /* the same MFMA tile code with launch boundaries as the only synchronisation
                                between workgroups (one launch per Sinkhorn pass; no kernel waits for
                                another workgroup): for a device that kernels of other streams share, where
                                the persistent kernels' grids may not become resident together (see "Waits
                                between workgroups" below).  d_k = d_v in {32, 64}, r <= 256; attention and
                                its backward, the [CLS] and cross variants; not lot_couplings */
} lot_path;

/*
 * Bytes of device workspace lot_attention_fwd (and its [CLS] variant) needs for this shape: the size
 * of what the kernels that LOT_PATH_AUTO selects really use -- a few megabytes on the tile kernels,
 * independent of n x r (the paper's "Rank and complexity": nothing of that size is formed).  The
 * _path form sizes a call whose path the caller forces (the plain kernels keep their n x r
 * intermediates in the workspace); lot_couplings_workspace_bytes does the same for lot_couplings /
 * lot_couplings_path (path = LOT_PATH_AUTO for the former).  Sizes depend on the device only through
 * its number of compute units (256 is assumed where no device is present).
 */
int lot_workspace_bytes(const lot_shape* shape, int iters, size_t* bytes_out);
int lot_workspace_bytes_path(const lot_shape* shape, int iters, int path, size_t* bytes_out);
int lot_couplings_workspace_bytes(const lot_shape* shape, int iters, int path, size_t* bytes_out);

/* out = LOTAttn(Q, K, V) as defined above (paper eq. (lotattn) with A = n * glued coupling). */
int lot_attention_fwd(const lot_shape* shape, const void* Q, const void* K, const void* V,
                      const float* Z, const float* beta, float eps, int iters, void* out,
                      void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * lot_attention_fwd for callers that cannot allocate device memory or hand one over: code under HIP
 * graph capture, tight serving loops, harnesses that forbid allocation.  Same operation, kernels,
 * arguments and rules as lot_attention_fwd with LOT_PATH_AUTO, minus the workspace: the scratch memory
 * is a fixed array inside the library, lot_static_scratch_bytes() = 32 MiB of device memory, which
 * every GPU that the library runs on holds until the process ends.  A shape whose kernels need more
 * (lot_workspace_bytes tells) is refused with LOT_ERR_SCRATCH before anything is launched; the
 * headline shape (B = 2, H = 8, n = 16384, r = 64) needs 18 MiB.  The call allocates and frees nothing
 * (no hipMalloc, no hipFree, no allocating library routine); the address of the array is looked up
 * once per device, at the first call with that device current.  The array needs no clearing between
 * calls (the kernels mark what they use per launch), but every call on one GPU shares it: calls that
 * overlap on one GPU (two streams, two threads) race and give undefined results -- serialise them, or
 * use lot_attention_fwd with workspaces of your own.
 */
size_t lot_static_scratch_bytes(void);
int lot_attention_fwd_static(const lot_shape* shape, const void* Q, const void* K, const void* V,
                             const float* Z, const float* beta, float eps, int iters, void* out,
                             void* hip_stream);

/*
 * Which kernels lot_attention_fwd_path would run for this shape on the current device (the choice between
 * the fused path's families depends on how many workgroups the device holds at once, so this asks the
 * device; nothing is launched).  The paper's cost model ("Rank and complexity": O(n d r + T n r)) is the
 * same for all of them; what differs is where the n x r kernel matrix exp(C/eps) lives between the
 * iterations, hence how many bytes a call moves:
 *   LOT_KERNELS_PLAIN           one plain kernel per step, everything through the workspace
 *   LOT_KERNELS_STREAMING       one persistent kernel that recomputes exp(C/eps) from Q, K in every pass
 *   LOT_KERNELS_KEPT_WORKGROUP  the same kernel keeping each workgroup's share of exp(C/eps) in registers
 *                               and LDS: Q, K, V are read once
 *   LOT_KERNELS_KEPT_WAVEFRONT  short sequences (up to 512 tokens; 1024 with bf16 I/O and at most 32 pivots): a
 *                               workgroup per problem, one, two or four wavefronts per side holding the side's whole
 *                               exp(C/eps) in their registers
 *   LOT_KERNELS_GROUPED         64 < r <= 256: pivots in groups of 64; one launch per step, or (short sequences:
 *                               few tiles per workgroup) everything in one launch
 */
typedef enum {
    LOT_KERNELS_PLAIN = 0,
    LOT_KERNELS_STREAMING = 1,
    LOT_KERNELS_KEPT_WORKGROUP = 2,
    LOT_KERNELS_KEPT_WAVEFRONT = 3,
    LOT_KERNELS_GROUPED = 4
} lot_kernels;
int lot_forward_kernels(const lot_shape* shape, int iters, int path, int* kernels_out);

/* Debug route: the two couplings themselves (paper: Gamma^(1) and Gamma^(2) in scaling form). */
int lot_couplings(const lot_shape* shape, const void* Q, const void* K,
                  const float* Z, const float* beta, float eps, int iters,
                  float* gamma1, float* gamma2,
                  void* workspace, size_t workspace_bytes, void* hip_stream);

/* Same two operations with the execution path chosen by the caller (lot_path). */
int lot_attention_fwd_path(const lot_shape* shape, const void* Q, const void* K, const void* V,
                           const float* Z, const float* beta, float eps, int iters, void* out,
                           void* workspace, size_t workspace_bytes, void* hip_stream, int path);
int lot_couplings_path(const lot_shape* shape, const void* Q, const void* K,
                       const float* Z, const float* beta, float eps, int iters,
                       float* gamma1, float* gamma2,
                       void* workspace, size_t workspace_bytes, void* hip_stream, int path);

/*
 * ViT variant with a [CLS] token (paper, "[CLS] under DS attention"): token 0 of every (batch, head)
 * is [CLS].  Rows 1 .. n-1 of out are the doubly-stochastic LOT attention AMONG tokens 1 .. n-1 (their
 * queries, keys and values only: uniform masses 1/(n-1), the same Z, beta, eps, iters); row 0 is a
 * standard softmax row over ALL n keys, alpha_j = softmax_j(beta_cls <q_0, k_j>), out_0 = sum_j
 * alpha_j v_j.  Same tensors, layout, workspace size (lot_workspace_bytes / _path of the full shape) and
 * rules as lot_attention_fwd; n >= 2, beta_cls > 0 (LOT_ERR_EPS otherwise).  The [CLS] polarisation
 * of the paper is not part of this entry point.
 */
int lot_attention_cls_fwd(const lot_shape* shape, const void* Q, const void* K, const void* V,
                          const float* Z, const float* beta, float eps, int iters, float beta_cls,
                          void* out, void* workspace, size_t workspace_bytes, void* hip_stream);
int lot_attention_cls_fwd_path(const lot_shape* shape, const void* Q, const void* K, const void* V,
                               const float* Z, const float* beta, float eps, int iters, float beta_cls,
                               void* out, void* workspace, size_t workspace_bytes, void* hip_stream, int path);

/*
 * Cross attention and non-uniform token masses (paper, "Empirical measures and pivot": queries and
 * keys are measures mu = sum_i p1_i delta_{q_i}, nu = sum_j p2_j delta_{k_j}, "typically" uniform;
 * the glued plan has marginals mu and nu; cross attention is named as in scope).
 *   Q [B,H,n_q,d_k], K [B,H,n_k,d_k], V [B,H,n_k,d_v], out [B,H,n_q,d_v] in io_dtype;
 *   mass_q [B,H,n_q], mass_k [B,H,n_k] fp32 device pointers, or NULL for uniform masses.  Masses are
 *   nonnegative and sum to one per (batch, head) (caller precondition, like beta); a token of mass
 *   zero is padding: it receives and sends nothing, whatever its row holds (finite values).
 * out = A V with A = Diag(mu)^-1 Gamma1 Diag(beta)^-1 Gamma2, the glued plan with renormalised rows
 * (for uniform masses and n_q = n_k this is n Gamma, i.e. lot_attention_fwd).  The row of a
 * zero-mass query is still defined (the limit of the formula) and written.
 * Execution paths as for lot_attention_fwd (lot_path): the tile kernels take d_k = d_v in {32, 64}
 * (r <= 64 the fused kernel, 64 < r <= 256 the grouped kernels); the plain kernels any shape; AUTO
 * prefers the tile kernels.  Workspace:
 * lot_cross_workspace_bytes (the kernels AUTO selects; _path for a forced path); lot_workspace_status applies.
 */
typedef struct {
    int32_t B, H;
    int32_t n_q, n_k;    /* query tokens, key/value tokens */
    int32_t d_k, d_v;
    int32_t r;
    int32_t io_dtype;
} lot_xshape;
int lot_cross_workspace_bytes(const lot_xshape* shape, int iters, size_t* bytes_out);
int lot_cross_workspace_bytes_path(const lot_xshape* shape, int iters, int path, size_t* bytes_out);
int lot_cross_attention_fwd(const lot_xshape* shape, const void* Q, const void* K, const void* V,
                            const float* Z, const float* beta, const float* mass_q, const float* mass_k,
                            float eps, int iters, void* out,
                            void* workspace, size_t workspace_bytes, void* hip_stream);
int lot_cross_attention_fwd_path(const lot_xshape* shape, const void* Q, const void* K, const void* V,
                                 const float* Z, const float* beta, const float* mass_q, const float* mass_k,
                                 float eps, int iters, void* out,
                                 void* workspace, size_t workspace_bytes, void* hip_stream, int path);

/*
 * Backward pass (paper, "Learning": the pivots, their masses and the projections are trained by
 * backpropagating through both Sinkhorn problems and the glued composition).  Given dO = dL/dO of
 * the forward call with the same inputs, eps and iters, writes
 *   dQ, dK [B,H,n,d_k], dV [B,H,n,d_v] in io_dtype (same layout as their tensors; dO as out),
 *   dZ [H,r,d_k], dbeta [H,r] in fp32, summed over the batch (Z and beta are shared across it).
 * These are the exact derivatives of the T-iteration forward function (every iteration of both
 * solves is differentiated, nothing is truncated); dbeta treats the r masses as free variables (no
 * projection onto the simplex).  The forward intermediates are recomputed inside; nothing has to be
 * saved from the forward call.  All gradient buffers are overwritten, not accumulated into.
 * Workspace: lot_attention_bwd_workspace_bytes (separate from, and larger than, the forward one: what the
 * kernels that AUTO selects use; lot_attention_bwd_workspace_bytes_path for a forced path);
 * contents on entry do not matter.  Same ownership, stream and error rules as the forward call;
 * gradient buffers must not alias the inputs, the workspace or each other.  iters <= 65536.
 * Two execution paths, chosen like the forward ones (lot_path): REFERENCE = one plain kernel per
 * step with the n x r intermediates in the workspace, any shape; FUSED = tiled MFMA kernels that
 * keep nothing of size n x r (d_k = d_v in {32, 64}; r <= 64, or 64 < r <= 256 with the pivots in groups
 * of 64; iters <= 64: the per-iteration tables live in a workgroup's local memory, and where those of all
 * groups do not fit there together the kernel that assembles dQ and dK runs once per run of groups, with
 * fp32 partial rows in the workspace in between; LOT_ERR_PATH beyond).  AUTO prefers
 * FUSED, except for fewer than 16 tokens and for r <= 2: there the rounding of the tile kernels'
 * contractions (2^-16 with fp32 I/O, bf16 operands with bf16 I/O) is not averaged out, or is magnified by
 * the cancellation in the gradient of two masses, and the plain kernels, exact to fp32 rounding, run instead.
 * Results are reproducible bit for bit on either path.  lot_workspace_status applies to this
 * workspace too (the FUSED path's forward sweep waits between workgroups when it runs as one kernel).
 * The FUSED path (r <= 64) rebuilds each tile's row-normalised kernels for all iterations with ONE shift
 * per row instead of a maximum per iteration, and checks every row sum against [2^-40, 2^40]: up to 16
 * iterations all of them are assembled at once and a workgroup that finds a sum outside is redone by a
 * second kernel, which goes iteration by iteration and re-shifts the rows of an iteration whose sum
 * leaves the range (lot_debug_set has knobs that make these rarely taken branches run on ordinary inputs).
 */
int lot_attention_bwd_workspace_bytes(const lot_shape* shape, int iters, size_t* bytes_out);
int lot_attention_bwd_workspace_bytes_path(const lot_shape* shape, int iters, int path, size_t* bytes_out);
int lot_attention_bwd(const lot_shape* shape, const void* Q, const void* K, const void* V,
                      const float* Z, const float* beta, float eps, int iters, const void* dO,
                      void* dQ, void* dK, void* dV, float* dZ, float* dbeta,
                      void* workspace, size_t workspace_bytes, void* hip_stream);
int lot_attention_bwd_path(const lot_shape* shape, const void* Q, const void* K, const void* V,
                           const float* Z, const float* beta, float eps, int iters, const void* dO,
                           void* dQ, void* dK, void* dV, float* dZ, float* dbeta,
                           void* workspace, size_t workspace_bytes, void* hip_stream, int path);

/*
 * Backward of lot_cross_attention_fwd (same inputs; dO [B,H,n_q,d_v]).  Writes dQ [B,H,n_q,d_k],
 * dK [B,H,n_k,d_k], dV [B,H,n_k,d_v] in io_dtype and dZ, dbeta in fp32 (summed over the batch).  The
 * masses are data (a padding mask), not differentiated; a key of mass zero receives exactly zero
 * gradient, a query of mass zero the gradient of its own output row.  Execution paths as for
 * lot_attention_bwd (FUSED: the tile kernels, r <= 64 in one register tile or 64 < r <= 256 in groups of
 * 64, within the same limits); AUTO prefers it.
 * Workspace: lot_cross_attention_bwd_workspace_bytes (the kernels AUTO selects; _path for a forced path);
 * contents on entry do not matter; lot_workspace_status applies.  Reproducible bit for bit on either path.
 */
int lot_cross_attention_bwd_workspace_bytes(const lot_xshape* shape, int iters, size_t* bytes_out);
int lot_cross_attention_bwd_workspace_bytes_path(const lot_xshape* shape, int iters, int path, size_t* bytes_out);
int lot_cross_attention_bwd(const lot_xshape* shape, const void* Q, const void* K, const void* V,
                            const float* Z, const float* beta, const float* mass_q, const float* mass_k,
                            float eps, int iters, const void* dO,
                            void* dQ, void* dK, void* dV, float* dZ, float* dbeta,
                            void* workspace, size_t workspace_bytes, void* hip_stream);
int lot_cross_attention_bwd_path(const lot_xshape* shape, const void* Q, const void* K, const void* V,
                                 const float* Z, const float* beta, const float* mass_q, const float* mass_k,
                                 float eps, int iters, const void* dO,
                                 void* dQ, void* dK, void* dV, float* dZ, float* dbeta,
                                 void* workspace, size_t workspace_bytes, void* hip_stream, int path);

/*
 * Backward of lot_attention_cls_fwd (same inputs, eps, iters, beta_cls; dO = dL/dout, all n rows).
 * dQ, dK, dV, dZ, dbeta as in lot_attention_bwd: rows 1 .. n-1 carry the gradient of the
 * doubly-stochastic part plus, in dK and dV, the share of the [CLS] row; row 0 of dQ is the gradient
 * of the [CLS] query, row 0 of dK and dV that of the [CLS] key and value (which only the softmax row
 * sees).  dbeta_cls [B,H] fp32: the derivative with respect to beta_cls PER (batch, head) problem --
 * sum it for a temperature shared by all of them.  Workspace: lot_attention_bwd_workspace_bytes (or _path) of
 * the full shape.  Paths and reproducibility as for lot_attention_bwd; the softmax row is one plain
 * kernel (one workgroup per problem) on either path.
 */
int lot_attention_cls_bwd(const lot_shape* shape, const void* Q, const void* K, const void* V,
                          const float* Z, const float* beta, float eps, int iters, float beta_cls, const void* dO,
                          void* dQ, void* dK, void* dV, float* dZ, float* dbeta, float* dbeta_cls,
                          void* workspace, size_t workspace_bytes, void* hip_stream);
int lot_attention_cls_bwd_path(const lot_shape* shape, const void* Q, const void* K, const void* V,
                               const float* Z, const float* beta, float eps, int iters, float beta_cls, const void* dO,
                               void* dQ, void* dK, void* dV, float* dZ, float* dbeta, float* dbeta_cls,
                               void* workspace, size_t workspace_bytes, void* hip_stream, int path);

/*
 * Waits between workgroups.  The fused forward kernel, the one-launch form of the grouped forward and the
 * tiled backward's forward sweep are persistent kernels whose workgroups exchange column sums; every such wait is bounded, and the grid
 * never exceeds what the device can hold at once.  A kernel of ANOTHER stream that occupies compute
 * units while one of these starts can still keep part of the grid from becoming resident; a wait then
 * gives up after its poll budget (seconds), every workgroup leaves, the rows of `out` that a leaving
 * workgroup owns (in the backward pass: dZ and dbeta) are filled with NaN so that the failure cannot
 * pass for a result, and the launch is marked in the first two words of the workspace.  The call itself has long returned
 * LOT_OK by then.  Three ways to see the mark:
 *   lot_workspace_status        synchronises the device and reads the words (debug).
 *   lot_workspace_status_async  enqueues, on the caller's stream, a copy of the two words to
 *                               host_words (pinned host memory, 16 bytes, owned by the caller); no
 *                               synchronisation.  Once the stream has passed that point,
 *   lot_status_words            (host only) turns the two words into LOT_OK or LOT_ERR_SYNC.
 * The next call on the same workspace is unaffected by an earlier failure.  A caller that shares the device
 * with other streams' kernels can avoid the waits altogether with LOT_PATH_STEPWISE (same results to
 * rounding, T + 4 launches instead of one); the Python autograd wrapper raises on a reported failure
 * and runs its later AUTO calls on that path.
 */
int lot_workspace_status(const void* workspace);
int lot_workspace_status_async(const void* workspace, unsigned long long* host_words, void* hip_stream);
int lot_status_words(const unsigned long long* host_words);

/*
 * Testing aids (for the library's own tests; no effect on results beyond rounding).  Process-wide;
 * value < 0 restores the default.  Nothing in the library reads the environment.
 *   LOT_KNOB_SPIN_LIMIT                poll budget of the bounded waits (default 2^21); 0 makes every
 *                                      wait give up at once: the kernels end early (every wavefront
 *                                      still exits) and the status words report the call
 *   LOT_KNOB_RESHIFT_BITS              0..40: narrows the backward assemble kernel's row-sum range to
 *                                      2^-bits .. 2^bits (0: practically every iteration re-shifts)
 *   LOT_KNOB_BWD_ASSEMBLE_BY_ITERATION non-zero: every workgroup through the iteration-by-iteration kernel
 *   LOT_KNOB_BWD_SWEEP_LAUNCHES        non-zero: the backward's forward sweep as one launch per pass
 *                                      (its form on a device that cannot hold the whole grid at once)
 *   LOT_KNOB_FWD_STREAMING             1: the fused forward re-reads Q and K in every pass (what it does for
 *                                      long sequences) also where the kernel matrix would fit on chip;
 *                                      2: the workgroup-level kept-matrix kernels wherever they fit (short
 *                                      sequences instead of the wavefront-per-side kernel; few iterations
 *                                      instead of the streaming kernel)
 *   LOT_KNOB_FWD_DRIFT_LIMIT           0..32: the forward kernels that keep exp(C/eps) on chip recompute it once
 *                                      the potentials have spread over more than this many binary orders
 *                                      (default 32; 0: in every iteration)
 *   LOT_KNOB_GROUPED_ONE_LAUNCH_TILES  the grouped forward (r > 64) runs as one launch when a workgroup has at
 *                                      most this many tiles of 32 tokens per side and the grid fits the device
 *                                      (default 8; 0: always one launch per step; large: wherever it fits)
 *   LOT_KNOB_BWD_SWEEP_RECOMPUTE       non-zero: the backward's forward sweep recomputes the similarities in every
 *                                      pass also where a wavefront has so few tiles that it would keep them in
 *                                      registers (the two forms differ by rounding, 1e-7; the one-launch-per-pass
 *                                      form always recomputes)
 * Returns LOT_OK, or LOT_ERR_SHAPE for an unknown knob.
 */
typedef enum {
    LOT_KNOB_SPIN_LIMIT = 0,
    LOT_KNOB_RESHIFT_BITS = 1,
    LOT_KNOB_BWD_ASSEMBLE_BY_ITERATION = 2,
    LOT_KNOB_BWD_SWEEP_LAUNCHES = 3,
    LOT_KNOB_FWD_STREAMING = 4,
    LOT_KNOB_FWD_DRIFT_LIMIT = 5,
    LOT_KNOB_GROUPED_ONE_LAUNCH_TILES = 6,
    LOT_KNOB_BWD_SWEEP_RECOMPUTE = 7,
    LOT_KNOB_COUNT_ = 8
} lot_knob;
int lot_debug_set(int knob, long long value);

/* Text for a lot_status; for LOT_ERR_HIP the text of the most recent HIP error on this thread. */
const char* lot_strerror(int code);

/* Library version: major * 10000 + minor * 100 + patch. */
int lot_version(void);

#ifdef __cplusplus
}
#endif
#endif /* LOT_H */
