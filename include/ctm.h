/*
 * ctm -- collapsed Taylor-mode PDE operators of a tanh MLP on one MI355X (gfx950).
 *
 * One call pushes a batch of points x[N,D], R first-order directional Taylor
 * coefficients per point and ONE summed highest-order coefficient through the
 * network and returns u[n] = f(x_n) together with
 *
 *     op[n] = scale * sum_{r=1..R} < d^K f(x_n), v_r^{(x)K} >        (Sec. 3.1, Eq. 5)
 *
 * one value per network output: for a network with C = d_L outputs u and op are [N, C]
 * and the operator acts on every output component (Sec. 3.2, Eq. 7), sharing the whole
 * propagation up to the last linear layer.  Wherever u, op (and gu, gop) are described as
 * [N] below, read [N, C] row-major for C > 1.
 *
 * for K = 2 (Laplacians, Sec. 3.2) or K = 4 (randomized biharmonic, Sec. 3.3).
 * The sum over r is taken inside the propagation ("collapsed", Sec. 3.1, Eq. 6):
 * every layer carries 1 + (K-1)R + 1 coefficient rows per point instead of 1 + K*R.
 *
 * The network is  f(x) = W_L act( ... act(W_1 x + b_1) ... ) + b_L  with C = d_L >= 1
 * outputs (1 in the paper's experiments), the activation after every layer but the last, and biases that
 * enter the 0-th coefficient only (App. H).  Coefficients are derivative-normalised
 * (Sec. 2: x(t) = sum_k t^k/k! x_k), so op is the K-th coefficient itself.
 *
 * Conventions
 *   - "dev" pointers are device memory of the GPU that is current when the call is
 *     made; "host" pointers are ordinary host memory.  All matrices are dense,
 *     row-major, with no padding; element type is the handle's storage type
 *     (double for CTM_F64, float for CTM_F32 and its bf16-MFMA variants).
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Calls
 *     only enqueue work on it and return; results are valid once the stream has
 *     reached that point.  No call synchronises the device except ctm_destroy_mlp.
 *   - Ownership: ctm_create_mlp copies (and re-packs) the weights, so the caller may
 *     free its own copies once `stream` has passed the call.  x, V, sigma, u, op and
 *     the workspace stay the caller's; the library allocates nothing in the
 *     operator calls.
 *   - Every function returns CTM_OK (0) or a negative ctm_status; it never throws or
 *     aborts.  Arguments are validated on the host before any GPU work is issued, and
 *     ctm_last_error() gives a readable message for the calling thread's last failure.
 *   - A handle is immutable: concurrent operator calls on one handle are fine as long
 *     as they use distinct workspaces.  It belongs to the device that was current at
 *     ctm_create_mlp; calls with another device current return CTM_ERR_UNSUPPORTED.
 */
#ifndef CTM_H
#define CTM_H

#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct ctm_mlp ctm_mlp; /* opaque */

typedef enum {
  CTM_F64 = 0,        /* fp64 storage, fp64 MFMA                                            */
  CTM_F32 = 1,        /* fp32 storage, fp32 MFMA (the benchmarked path)                     */
  CTM_F32_BF16X3 = 2, /* fp32 storage; GEMMs on the bf16 matrix cores with every operand split
                         into hi + lo bf16 parts (3 MFMAs per product, fp32 accumulate)      */
  CTM_F32_BF16 = 3,   /* fp32 tensors at the boundary; GEMM inputs rounded to bf16 (1 MFMA, fp32 accumulate;
                         the workspace blocks between layers are kept in bf16)                */
  CTM_DTYPE_RANGE_ = 0x7fffffff /* not a dtype: widens the enum to int, so that an unknown value passed in by a
                                   caller is an ordinary value the library can refuse (CTM_ERR_DTYPE)           */
} ctm_dtype;

typedef enum {
  CTM_ACT_TANH = 0,
  CTM_ACT_IDENTITY = 1, /* linear network: every operator is exactly 0 (a test hook)          */
  CTM_ACT_SIN = 2,      /* sin, the elementwise example of the paper's graph-rewrite appendix  */
  CTM_ACT_RANGE_ = 0x7fffffff /* not an activation: widens the enum to int (see CTM_DTYPE_RANGE_)      */
} ctm_act;

typedef enum {
  CTM_OK = 0,
  CTM_ERR_NULL = -1,        /* a required pointer is NULL                           */
  CTM_ERR_SHAPE = -2,       /* a size or stride is out of range or inconsistent     */
  CTM_ERR_DTYPE = -3,       /* unknown dtype / activation enum value                */
  CTM_ERR_UNSUPPORTED = -4, /* valid request this build does not cover              */
  CTM_ERR_WORKSPACE = -5,   /* workspace smaller than ctm_workspace_bytes() says    */
  CTM_ERR_ALIGN = -6,       /* a pointer is not aligned as the call requires        */
  CTM_ERR_ALLOC = -7,       /* device allocation failed (ctm_create_mlp only)       */
  CTM_ERR_HIP = -8          /* a HIP runtime call failed; text in ctm_last_error()  */
} ctm_status;

/*
 * Build a handle for an MLP with n_layers linear layers (n_layers >= 2, i.e. at least one
 * hidden layer) of widths dims[0] = D, ..., dims[n_layers] = C   (Sec. 4 setup; App. H model).
 *   dims  host, n_layers + 1 ints, all >= 1; dims[n_layers] = C, the number of outputs, at most 1024
 *   W     host array of n_layers dev pointers; W[l] is [dims[l+1], dims[l]] row-major
 *   b     host array of n_layers dev pointers to [dims[l+1]]; the array or any entry may
 *         be NULL, meaning a zero bias
 * The weights are copied into the library's own zero-padded tile layout on `stream`.
 * On failure *out is set to NULL.
 */
int ctm_create_mlp(int n_layers, const int *dims, const void *const *W, const void *const *b,
                   ctm_dtype dtype, ctm_act act, void *stream, ctm_mlp **out);

/* Waits for the device, then frees the handle's device memory.  NULL is allowed. */
int ctm_destroy_mlp(ctm_mlp *mlp);

/*
 * Coefficient rows carried per point by collapsed Taylor mode of order K with R
 * directions: 1 + (K-1)*R + 1 (Sec. 3.1).  K must be 2 or 4, R >= 1; returns -1 otherwise.
 */
long ctm_rows_per_point(int K, int R);

/*
 * Bytes of device workspace an operator call of order K (2 or 4) on N points with R
 * directions needs.  Returns 0 on invalid arguments (and sets ctm_last_error()).
 * The workspace must be 256-byte aligned; its contents are scratch.
 */
size_t ctm_workspace_bytes(const ctm_mlp *mlp, int K, long N, int R);

/*
 * Second-order operator  op[n] = scale * sum_r v_r^T (Hessian f)(x_n) v_r      (Sec. 3.2, Eq. 7)
 *   x       dev [N, D]
 *   V       dev directions, or NULL for the standard basis e_1..e_D (then R must equal D):
 *           the exact Laplacian.  v_point_stride = 0: V is [R, D], shared by all points;
 *           v_point_stride = R*D: V is [N, R, D], own directions per point.
 *   scale   1 for exact operators, 1/S for the S-sample randomized Laplacian; applied to
 *           the final scalar only
 *   u, op   dev [N] outputs; either may be NULL if not wanted
 * Any R >= 1 is accepted; direction sets too large for one tile are processed in several
 * passes whose partial sums are added in a fixed order.
 */
int ctm_laplacian(const ctm_mlp *mlp, const void *x, long N, const void *V, int R,
                  long v_point_stride, double scale, void *u, void *op, void *workspace,
                  size_t workspace_bytes, void *stream);

/*
 * ctm_laplacian for callers that cannot allocate device memory at all: code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc.  Same arguments and results (bit for bit, the same kernels
 * run) as ctm_laplacian, but the workspace is a device array built into the library, CTM_STATIC_SCRATCH_BYTES
 * long; every GPU the library runs on holds its copy until the process ends.  The call allocates nothing and
 * frees nothing; the caller still owns x, V, u and op.
 *   - A request with ctm_workspace_bytes(mlp, 2, N, R) > CTM_STATIC_SCRATCH_BYTES returns CTM_ERR_WORKSPACE
 *     and launches nothing (the benchmark network with basis directions fits 206 points; split larger
 *     batches or use ctm_laplacian).
 *   - All calls on one GPU share that GPU's array: calls that overlap in time on one GPU (two streams, two
 *     threads) race.  Calls in stream order on one stream are fine; the array keeps the previous call's
 *     contents and every element a call reads is written by that call first, so nothing needs clearing.
 *   - The first call on a device looks up the array's address (hipGetSymbolAddress); make one call before
 *     starting a graph capture.
 */
#define CTM_STATIC_SCRATCH_BYTES (64u << 20)
int ctm_laplacian_static(const ctm_mlp *mlp, const void *x, long N, const void *V, int R,
                         long v_point_stride, double scale, void *u, void *op, void *stream);

/*
 * Weighted Laplacian  op[n] = Tr(sigma sigma^T Hessian f(x_n)) = sum_k s_k^T H s_k     (Sec. 3.2, Eq. 8)
 *   sigma   dev [D, K] row-major, shared by all points; the directions are its K columns
 * Same as ctm_laplacian with V = sigma^T, shared, scale = 1.
 */
int ctm_weighted_laplacian(const ctm_mlp *mlp, const void *x, long N, const void *sigma, int K,
                           void *u, void *op, void *workspace, size_t workspace_bytes,
                           void *stream);

/*
 * Weighted Laplacian with a point-dependent sigma and / or Monte-Carlo directions       (Sec. 3.2, Eq. 8)
 *   sigma   dev; sigma_point_stride = 0: [D, K] shared; = D*K: [N, D, K], sigma depends on the point
 *   V       dev random vectors in R^K; v_point_stride = 0: [S, K] shared; = S*K: [N, S, K] per point.
 *           op[n] = (1/S) sum_s (sigma_n v_{n,s})^T H(x_n) (sigma_n v_{n,s})    (stochastic case)
 *           V = NULL with S = 0: the exact operator Tr(sigma_n sigma_n^T H(x_n)), directions = columns of sigma_n
 * The directions sigma_n v_{n,s} are formed on the device in the tail of the workspace.
 * Workspace: ctm_weighted_laplacian_rand_workspace_bytes(...) bytes (0 on invalid arguments), 256-byte aligned.
 */
size_t ctm_weighted_laplacian_rand_workspace_bytes(const ctm_mlp *mlp, long N, int K, int S,
                                                   long sigma_point_stride, long v_point_stride);
int ctm_weighted_laplacian_rand(const ctm_mlp *mlp, const void *x, long N, const void *sigma, int K,
                                long sigma_point_stride, const void *V, int S, long v_point_stride,
                                void *u, void *op, void *workspace, size_t workspace_bytes, void *stream);

/*
 * Randomized biharmonic  op[n] = 1/(3S) * sum_s < d^4 f(x_n), v_s^{(x)4} >         (Sec. 3.3, Eq. 9)
 * by collapsed 4th-order Taylor mode (1 + 3S + 1 rows per point).  V and
 * v_point_stride as in ctm_laplacian (V must not be NULL).  The estimator is unbiased
 * for standard-normal directions only; the call itself accepts any V.
 */
int ctm_biharmonic_rand(const ctm_mlp *mlp, const void *x, long N, const void *V, int S,
                        long v_point_stride, void *u, void *op, void *workspace,
                        size_t workspace_bytes, void *stream);

/*
 * Gradients with respect to the weights ("differentiable" evaluation, Sec. 4) for second-order operators.
 *
 * ctm_laplacian_fwd computes the same (u, op) as ctm_laplacian (collapsed order-2 Taylor mode) and records, in
 * the caller's `tape`, what the reverse pass needs: the input coefficient block and, per hidden layer, the
 * pre-activation rows and the output rows.  Any R >= 1: direction sets too large for one tile are split into passes,
 * each with a tape of its own (ctm_tape_bytes counts them all), and the reverse pass adds the gradients of the passes
 * in pass order.  CTM_F32 and CTM_F64 handles.
 *   tape    dev, ctm_tape_bytes(mlp, N, R) bytes (0 on invalid arguments), 256-byte aligned
 *
 * ctm_laplacian_bwd takes dL/du and dL/dop of a scalar L and the tape of the matching forward call (same mlp
 * weights, N, R, scale) and writes dL/dW_l and dL/db_l:
 *   gu, gop   dev [N], either may be NULL (= zeros)
 *   gW, gb    host arrays of n_layers dev pointers, gW[l] is [dims[l+1], dims[l]] row-major, gb[l] is [dims[l+1]];
 *             the arrays or single entries may be NULL (gradient not wanted).  Outputs are overwritten, not
 *             accumulated; all sums over points use fixed partitions and orders (bitwise reproducible).
 *   workspace dev, ctm_backward_workspace_bytes(mlp, N, R) bytes, 256-byte aligned
 * Per hidden layer it runs: the cotangent GEMM Zbar W fused with the reverse of the activation rule (the same
 * stacked-GEMM kernel), the weight gradient Zbar^T H over all N * rho rows, and the bias gradient.
 *
 * ctm_update_mlp re-packs new weights (same shapes) into an existing handle, e.g. after an optimizer step.
 * The reverse pass reads the weights from the handle, so a *_bwd call must find the weights its *_fwd call ran with:
 * a handle remembers, per tape address, which update of its weights the recording forward saw, and a *_bwd call
 * on a tape recorded before the latest ctm_update_mlp returns CTM_ERR_UNSUPPORTED (run forward again).  Calls
 * that replace the weights must not overlap with operator calls on the same handle.
 */
size_t ctm_tape_bytes(const ctm_mlp *mlp, long N, int R);
size_t ctm_backward_workspace_bytes(const ctm_mlp *mlp, long N, int R);
int ctm_laplacian_fwd(const ctm_mlp *mlp, const void *x, long N, const void *V, int R, long v_point_stride,
                      double scale, void *u, void *op, void *tape, size_t tape_bytes, void *stream);
int ctm_laplacian_bwd(const ctm_mlp *mlp, long N, int R, double scale, const void *tape, size_t tape_bytes,
                      const void *gu, const void *gop, void *const *gW, void *const *gb, void *workspace,
                      size_t workspace_bytes, void *stream);
int ctm_update_mlp(ctm_mlp *mlp, const void *const *W, const void *const *b, void *stream);

/*
 * The same pair of calls for the randomized biharmonic (Sec. 3.3, Eq. 9; "differentiable" evaluation, Sec. 4):
 * ctm_biharmonic_rand_fwd computes the (u, op) of ctm_biharmonic_rand by collapsed order-4 Taylor mode and
 * records the tape; ctm_biharmonic_rand_bwd runs the reverse of the order-4 rule (it needs the fifth derivative
 * of the activation) and writes dL/dW_l, dL/db_l.  Any S >= 1 (several passes beyond S = 84, as above).  Arguments as in the Laplacian pair;
 * the scale 1/(3S) is implied.  V must not be NULL.
 */
size_t ctm_biharmonic_tape_bytes(const ctm_mlp *mlp, long N, int S);
size_t ctm_biharmonic_backward_workspace_bytes(const ctm_mlp *mlp, long N, int S);
int ctm_biharmonic_rand_fwd(const ctm_mlp *mlp, const void *x, long N, const void *V, int S, long v_point_stride,
                            void *u, void *op, void *tape, size_t tape_bytes, void *stream);
int ctm_biharmonic_rand_bwd(const ctm_mlp *mlp, long N, int S, const void *tape, size_t tape_bytes, const void *gu,
                            const void *gop, void *const *gW, void *const *gb, void *workspace,
                            size_t workspace_bytes, void *stream);

/*
 * And for the exact biharmonic (Sec. 3.3, Eq. 12; "differentiable" evaluation, Sec. 4): the forward records one
 * order-4 tape per direction family of the interpolation formula, the reverse pass runs once per family and adds
 * the three contributions in a fixed order (u enters through the first).  Any D: families of more than 84 directions
 * (D >= 10) run in several passes.  Arguments as in the pairs above.
 */
size_t ctm_biharmonic_exact_tape_bytes(const ctm_mlp *mlp, long N);
size_t ctm_biharmonic_exact_backward_workspace_bytes(const ctm_mlp *mlp, long N);
int ctm_biharmonic_exact_fwd(const ctm_mlp *mlp, const void *x, long N, void *u, void *op, void *tape,
                             size_t tape_bytes, void *stream);
int ctm_biharmonic_exact_bwd(const ctm_mlp *mlp, long N, const void *tape, size_t tape_bytes, const void *gu,
                             const void *gop, void *const *gW, void *const *gb, void *workspace,
                             size_t workspace_bytes, void *stream);

/*
 * The same sums computed by STANDARD (un-collapsed) Taylor mode, for comparison only: every direction
 * carries its own order-K coefficient through the network (1 + K*R rows per point, Sec. 3.1) and the sum
 * over directions is taken after the last layer.  K = 2 or 4; other arguments as in ctm_laplacian
 * (K = 4: op = scale * sum_r <d^4 f, v_r^4>, pass scale = 1/(3S) for the biharmonic estimator).
 * Mathematically equal to the collapsed calls; it exists to measure what collapsing saves on this GPU.
 * Workspace: ctm_workspace_bytes_standard(mlp, K, N, R).
 */
size_t ctm_workspace_bytes_standard(const ctm_mlp *mlp, int K, long N, int R);
int ctm_taylor_standard(const ctm_mlp *mlp, int K, const void *x, long N, const void *V, int R,
                        long v_point_stride, double scale, void *u, void *op, void *workspace,
                        size_t workspace_bytes, void *stream);

/*
 * Exact biharmonic  op[n] = sum_{d1,d2} d^4 f / dx_{d1}^2 dx_{d2}^2 (x_n)          (Sec. 3.3, Eq. 9 exact case)
 * by interpolation with three collapsed families of 4-jets (Sec. 3.3 Eq. 12; App. E.1, last display):
 *   op = 1/24 [ (2 D g40 + 2 g31 + g22) sum_d <d^4 f,(4 e_d)^4> + 2 g31 sum_{d1 != d2} <d^4 f,(3 e_d1 + e_d2)^4>
 *               + 2 g22 sum_{d1 < d2} <d^4 f,(2 e_d1 + 2 e_d2)^4> ],   g_j = gamma_{(2,2), j}.
 * The families have D, D(D-1) and D(D-1)/2 directions; they are generated on the device into the
 * workspace and run as shared-direction order-4 calls whose results are added in this order.
 * Workspace: ctm_biharmonic_exact_workspace_bytes(mlp, N) bytes (0 on invalid arguments), 256-byte aligned.
 */
size_t ctm_biharmonic_exact_workspace_bytes(const ctm_mlp *mlp, long N);
int ctm_biharmonic_exact(const ctm_mlp *mlp, const void *x, long N, void *u, void *op, void *workspace,
                         size_t workspace_bytes, void *stream);

/*
 * Interpolation coefficient gamma_{i,j} of the mixed-partial reconstruction (App. E, the coefficient
 * definition with generalised binomials), as an exact fraction num/den in lowest terms (den > 0).
 *   I     number of distinct directions (1..4); i, j: host arrays of I non-negative ints with
 *         |i| = |j| in 1..8
 * Pure host arithmetic.
 */
int ctm_interpolation_gamma(int I, const int *i, const int *j, long long *num, long long *den);

/*
 * Host-side description of how an order-K, R-direction call is tiled: points per tile,
 * 16-row MFMA blocks per tile, directions in the first (largest) pass and number of
 * passes, for a batch large enough to fill the GPU (small batches may get shorter tiles).
 * Pure host logic (no GPU needed); any output pointer may be NULL.
 */
int ctm_tile_plan(ctm_dtype dtype, int K, int R, int *points_per_tile, int *row_blocks,
                  int *dirs_per_pass, int *n_passes);

/* Message for the calling thread's most recent failing call ("" if none). */
const char *ctm_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* CTM_H */
