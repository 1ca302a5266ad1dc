/*
 * sparse_topk.h -- C ABI of the MI355X (gfx950) library for the p-norm-regularised, differentiable
 * and sparse top-k operators of "Fast, Differentiable and Sparse Top-k: a Convex Analysis
 * Perspective" (Sander, Puigcerver, Djolonga, Peyre, Blondel; ICML 2023).
 *
 * The operators (paper Sec. 4, "Differentiable and sparse top-k operators"), per row x in R^n:
 *
 *   relaxed top-k mask          y = grad_1 f_{phi,R}(x, 1_k)  with phi(x) = x
 *   relaxed top-k in magnitude  y = grad_1 f_{phi,R}(x, 1_k)  with phi(x) = x^2 / 2
 *
 * where 1_k = (1,..,1,0,..,0) has k ones (Eq. (topk_mask)), R(y) = (lambda / p) * sum_i |y_i|^p,
 * and by Prop. 2 (relaxed operator)  y = grad R*(x - u*),  u* = argmin_u R*(x - u) + f_phi(u, 1_k).
 * u* is obtained exactly through the reduction to isotonic optimisation (Prop. 5 for phi = x,
 * Prop. 6 for phi = x^2/2): sort x (or |x|) in descending order, solve
 *     v* = argmin_{v_1 >= ... >= v_n} sum_i r*(s_i - v_i) + w_i phi(v_i)       (Eq. (isotonic_separable))
 * and un-permute (times sign(x) for the magnitude operator).  The Jacobian-vector products use
 * the closed form of Prop. 7 (differentiation).  Only p = 2 and p = 4/3 have closed-form pooling
 * steps (Sec. 7, "Sensitivity to the choice of p") and only those are accepted.
 *
 * Conventions shared by all entry points
 *   - Every data pointer is a DEVICE pointer (HBM of the current HIP device), owned by the
 *     caller, to a row-major contiguous [rows][n] array: float for values, int32_t for
 *     permutations.  Outputs must not alias inputs or each other.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Calls only enqueue
 *     work on that stream; they never synchronise with the host and never allocate.
 *   - Sorting is descending; equal values keep ascending original index; -0.0f counts as +0.0f.
 *   - Merges of the pool-adjacent-violators partition happen on strict violations only, so at a
 *     kink of the p = 2 operator the derivative taken is the one of the un-merged side.
 *   - 1 <= n < 2^30, 0 <= k <= n, lambda > 0 and finite, rows >= 0 (rows == 0 is a no-op).
 *     k == 0 gives all zeros; k == n gives all ones (mask) or x / (1 + lambda) (magnitude, p = 2).
 *   - NaN or infinite inputs are a precondition violation (the output is then unspecified, but
 *     no out-of-bounds access happens).
 *   - Return value: TOPK_OK, or a negative TOPK_ERR_* code, in which case nothing was enqueued.
 *   - Long rows (above 2048 elements; above TOPK_SHORT_ROW_MAX for top-k in magnitude with
 *     p = 4/3) go through HBM scratch memory that the caller provides: query
 *     topk_workspace_bytes(), hand the buffer over with topk_set_workspace().
 *     The workspace is process-global: calls that use it must not overlap in time (different
 *     streams, or host threads) -- they would race on it.
 */
#ifndef SPARSE_TOPK_H_
#define SPARSE_TOPK_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
  TOPK_OK = 0,
  TOPK_ERR_INVALID = -1,        /* rows < 0, n < 1, n >= 2^30, k < 0, k > n, lambda <= 0 or non-finite */
  TOPK_ERR_NULL = -2,           /* a required pointer is NULL */
  TOPK_ERR_UNSUPPORTED_P = -3,  /* p is neither 2 nor 4/3 */
  TOPK_ERR_WORKSPACE = -4,      /* long rows and the registered workspace is missing or too small */
  TOPK_ERR_LAUNCH = -5,         /* the HIP runtime refused a launch (see hipGetLastError) */
  TOPK_ERR_STATIC_SCRATCH = -6  /* topk_mask_jvp_static: the shape needs more scratch than
                                   TOPK_STATIC_SCRATCH_BYTES */
};

/* Operator codes for topk_workspace_bytes(). */
enum {
  TOPK_OP_MASK_FWD = 0,
  TOPK_OP_MASK_JVP = 1,
  TOPK_OP_MAG_FWD = 2,
  TOPK_OP_MAG_JVP = 3,
  TOPK_OP_ARGSORT = 4,
  TOPK_OP_SIGNED_MASK = 5,   /* topk_signed_mask_fwd and _jvp */
  TOPK_OP_MASKED_VALUE = 6,  /* topk_masked_value_fwd and _jvp */
  TOPK_OP_GENERAL = 7,       /* topk_general_fwd and _jvp */
  TOPK_OP_MASK_SPARSE = 8    /* topk_mask_sparse_fwd */
};

/* phi of topk_general_*: phi(x) = x (mask-like operators) or phi(x) = x^2 / 2 (in magnitude). */
enum {
  TOPK_PHI_IDENTITY = 0,
  TOPK_PHI_HALF_SQUARE = 1
};

/* Rows up to this length are handled by one wavefront in registers by every entry point (no
 * workspace needed); the dense operators take rows of up to 2048 elements that way, except
 * top-k in magnitude with p = 4/3. */
#define TOPK_SHORT_ROW_MAX 1024
/* Longest row of topk_general_*: above TOPK_SHORT_ROW_MAX one workgroup solves a sorted row. */
#define TOPK_GENERAL_ROW_MAX 131072

/*
 * Relaxed top-k mask, forward (phi(x) = x; Prop. 2 + Prop. 5; pooling steps from Sec. 5
 * "Example" for p = 2 and App. "Subproblem derivation" for p = 4/3).
 *   theta [rows][n] in,  out [rows][n] out: values in [0, 1] summing to k per row, with exact
 *   0.0f below the pooled block and exact 1.0f above it.
 *   p: 2.0 or 4.0/3.0 (matched with a small tolerance).  lambda: regularisation strength.
 */
int topk_mask_fwd(const float* theta, int64_t rows, int64_t n, int64_t k, double p, double lambda,
                  float* out, void* stream);

/*
 * Jacobian-vector product of the relaxed top-k mask (Prop. 7, differentiation), fused with the
 * forward pass: jvp_out = (d y / d theta) . tangent.  `out` may be NULL (JVP only); when given it
 * receives the same values as topk_mask_fwd.  The sort and the block are recomputed (the call is
 * stateless).
 */
int topk_mask_jvp(const float* theta, const float* tangent, int64_t rows, int64_t n, int64_t k,
                  double p, double lambda, float* out, float* jvp_out, void* stream);

/*
 * Relaxed top-k in magnitude, forward (phi(x) = x^2/2; Prop. 2 + Prop. 6): sort |x|, solve on the
 * non-negative monotone cone, restore the signs.  Pruned entries are +0.0f.  sign(0) = 0.
 * p = 2: pooling step of Sec. 5 "Example", gamma = sum_B s / (|B| + lambda m); kept entries
 * before the pooled block come out as x / (1 + lambda).
 * p = 4/3: pooling step of App. "Subproblem derivation" with phi = x^2/2: gamma is the root of
 * sum_B (gamma - s_i)^3 + lambda^3 m gamma = 0 (m = kept positions in B); kept entries before the
 * block come out as sign(x) g with g the root of (g - |x|)^3 + lambda^3 g = 0.
 */
int topkmag_fwd(const float* x, int64_t rows, int64_t n, int64_t k, double p, double lambda,
                float* out, void* stream);

/*
 * topk_mask_jvp for callers that cannot allocate or register device memory: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, results (bit for
 * bit) and errors as topk_mask_jvp, but rows that need scratch (above 2048 elements) use a scratch
 * array that is part of the library's device image instead of the registered workspace; the
 * call allocates nothing, frees nothing and ignores topk_set_workspace.
 *   - Limit: topk_workspace_bytes(TOPK_OP_MASK_JVP, rows, n, k, p) <= TOPK_STATIC_SCRATCH_BYTES
 *     (about rows * n <= 3.6 million elements); larger shapes return TOPK_ERR_STATIC_SCRATCH
 *     with nothing enqueued.  Rows of up to 2048 elements need no scratch and have no such
 *     limit.
 *   - Every GPU the library is used on holds its own copy of the array (TOPK_STATIC_SCRATCH_BYTES
 *     of device memory, for the life of the process); the first call on a device looks its
 *     address up (make that call outside a stream capture).
 *   - All calls on one GPU share that GPU's array and nothing in it needs to start at zero, but
 *     two calls that overlap in time on one GPU (different streams, or threads) race on it:
 *     serialise them on one stream.
 */
#define TOPK_STATIC_SCRATCH_BYTES (64u << 20)
int topk_mask_jvp_static(const float* theta, const float* tangent, int64_t rows, int64_t n,
                         int64_t k, double p, double lambda, float* out, float* jvp_out,
                         void* stream);

/* JVP of the relaxed top-k in magnitude (Prop. 7, case phi = x^2/2), fused with the forward pass;
 * `out` may be NULL. */
int topkmag_jvp(const float* x, const float* tangent, int64_t rows, int64_t n, int64_t k,
                double p, double lambda, float* out, float* jvp_out, void* stream);

/*
 * Vector-Jacobian products, for reverse-mode differentiation: vjp_out = cotangent . (d y / d x).
 * Both operators are gradients in their first argument of the convex function f_{phi,R}(., 1_k)
 * (Prop. 2: y = grad_1 f_{phi,R}(x, 1_k)), so their Jacobians are symmetric wherever they exist
 * (for the magnitude operator J = diag(sign x) J_s diag(sign x) with J_s symmetric), and the
 * closed form of Prop. 7 serves both directions: these calls compute exactly what the *_jvp calls
 * compute, with the cotangent in the place of the tangent.  Same arguments, layout and errors;
 * `out` may be NULL.
 */
int topk_mask_vjp(const float* theta, const float* cotangent, int64_t rows, int64_t n, int64_t k,
                  double p, double lambda, float* out, float* vjp_out, void* stream);
int topkmag_vjp(const float* x, const float* cotangent, int64_t rows, int64_t n, int64_t k,
                double p, double lambda, float* out, float* vjp_out, void* stream);

/*
 * Relaxed top-k mask in compact form, e.g. for dispatching tokens to the selected experts (Sec. 6,
 * sparse mixture of experts): the operator's output is exactly zero below the pooled block, so a
 * row is described by its non-zeros.  Per row, in descending order of theta (ties by ascending
 * index): idx_out[r][j] = index of the j-th largest entry, val_out[r][j] = its mask value, for
 * j < min(nnz_out[r], max_nnz); the remaining slots hold -1 / 0.0f.  nnz_out[r] is the number of
 * non-zeros (k <= nnz <= n for k >= 1); if it exceeds max_nnz the list was cut off.
 *   theta [rows][n] in; idx_out (int32) and val_out (float) [rows][max_nnz], nnz_out (int32) [rows]
 *   out.  1 <= max_nnz <= n.  Rows above
 *   TOPK_SHORT_ROW_MAX need the workspace of TOPK_OP_MASK_SPARSE, and their lists are ordered
 *   differently: first the entries that lie above everything that can pool (value exactly 1), in
 *   ascending index order, then the remaining non-zeros in descending order of theta.
 *   Other arguments and errors as topk_mask_fwd.
 */
int topk_mask_sparse_fwd(const float* theta, int64_t rows, int64_t n, int64_t k, double p,
                         double lambda, int64_t max_nnz, int32_t* idx_out, float* val_out,
                         int32_t* nnz_out, void* stream);

/*
 * The relaxed operators for a general weight vector (Sec. 4: y_{phi,R}(x, w) = grad_1
 * f_{phi,R}(x, w), Prop. 2; reductions of Prop. 5 / Prop. 6; full PAV partition of App. "PAV
 * algorithm"; JVP in x by Prop. 7).  With the LP forms of Sec. 3 this gives relaxed ranks
 * (input -theta, w = (n, .., 1)), relaxed sorts (input (n, .., 1), w = sort(theta), one weight
 * row per row) and partial ranks; w = 1_k reproduces topk_mask_* / topkmag_*.
 *   x [rows][n] in.  w: weights by SORTED position, non-increasing (w_1 >= ... >= w_n >= 0; not
 *   checked, the result is unspecified otherwise): [n] shared by all rows when w_stride == 0,
 *   [rows][n] when w_stride == n (anything else: TOPK_ERR_INVALID).  phi: a TOPK_PHI_* code.
 *   out, jvp_out [rows][n] out (out may be NULL in the *_jvp call).
 *   Rows up to TOPK_GENERAL_ROW_MAX elements (TOPK_ERR_INVALID beyond).  Up to TOPK_SHORT_ROW_MAX
 *   elements the lanes of a wavefront build the partition of a row together and no workspace is
 *   needed; longer rows are sorted completely and then solved by one workgroup each, with
 *   topk_workspace_bytes(TOPK_OP_GENERAL, rows, n, 0, p) bytes of workspace (TOPK_ERR_WORKSPACE
 *   without).  The partition is built in rounds that remove all violating block boundaries at
 *   once; rows on which only one boundary violates at a time fall back to the sequential walk of
 *   the block stack and are slow.  Other arguments and errors as topk_mask_fwd / topk_mask_jvp.
 */
int topk_general_fwd(const float* x, const float* w, int64_t w_stride, int64_t rows, int64_t n,
                     int phi, double p, double lambda, float* out, void* stream);
int topk_general_jvp(const float* x, const float* w, int64_t w_stride, const float* tangent,
                     int64_t rows, int64_t n, int phi, double p, double lambda, float* out,
                     float* jvp_out, void* stream);

/*
 * Relaxed top-k mask for p = 2 by Dykstra's alternating projection algorithm (Sec. 5, Alg. 1)
 * instead of the exact solve: `iters` rounds of projections onto the even-pair and odd-pair
 * constraint sets, started from s - lambda 1_k on the sorted row (the linear term enters once).
 * An approximation that converges to topk_mask_fwd's result as iters grows (the paper uses 100);
 * iters == 0 returns the hard top-k mask.  The alternative solver for comparisons: rows up to
 * TOPK_SHORT_ROW_MAX elements only (TOPK_ERR_INVALID beyond, and for iters < 0), float64
 * iterates in registers, no workspace.  Other arguments and errors as topk_mask_fwd.
 */
int topk_mask_dykstra_fwd(const float* theta, int64_t rows, int64_t n, int64_t k, double lambda,
                          int iters, float* out, void* stream);

/*
 * Two more operators on the magnitudes, both built on the relaxed top-k mask m(.) of |x|.
 *
 * Signed relaxed top-k mask (phi(x) = |x|; Sec. 4, "Connection with k-support and OWL norms":
 * with this phi the operator in magnitude becomes a signed top-k mask).  By the reduction of
 * Prop. 6 the isotonic problem is the mask's on s = sort(|x|) with the constraint v >= 0, handled
 * by truncation (Sec. 5), so per element y = sign(x) min(m_i, grad r*(|x_i|)): where the
 * truncation is active (magnitudes below about lambda) y_i = grad r*(x_i) = sign(x_i) (|x_i| /
 * lambda)^(q-1) and dy_i = hess r*(x_i) t_i, elsewhere y = sign(x) o m(|x|) and
 * dy = sign(x) o J_m (sign(x) o t).  sign(0) = 0.
 *
 * Masked value (Sec. 7, "Advantage of the non-linearity": the alternative top-k in magnitude):
 * y = x o m(|x|), dy = t o m(|x|) + x o J_m (sign(x) o t).
 *
 *   x, tangent [rows][n] in; out, jvp_out [rows][n] out (out is required by the *_jvp calls too).
 *   Rows of 3..2048 elements run in one kernel and need no workspace; other row lengths need two
 *   float arrays of the input's size, plus the mask's own for long rows:
 *   topk_workspace_bytes(TOPK_OP_SIGNED_MASK / TOPK_OP_MASKED_VALUE).
 *   Otherwise the arguments, p values and errors of topk_mask_fwd / topk_mask_jvp.
 */
int topk_signed_mask_fwd(const float* x, int64_t rows, int64_t n, int64_t k, double p,
                         double lambda, float* out, void* stream);
int topk_signed_mask_jvp(const float* x, const float* tangent, int64_t rows, int64_t n, int64_t k,
                         double p, double lambda, float* out, float* jvp_out, void* stream);
int topk_masked_value_fwd(const float* x, int64_t rows, int64_t n, int64_t k, double p,
                          double lambda, float* out, void* stream);
int topk_masked_value_jvp(const float* x, const float* tangent, int64_t rows, int64_t n, int64_t k,
                          double p, double lambda, float* out, float* jvp_out, void* stream);

/*
 * Smooth top-k loss (Sec. 6, "Smooth top-k loss"): the Fenchel-Young loss of the relaxed top-k
 * mask, per row
 *     loss = f_{phi,R}(theta, 1_k) - <theta, target>,   phi(x) = x,
 * and its gradient in theta, grad = y - target with y the mask of topk_mask_fwd (Prop. 2:
 * y = grad_1 f_{phi,R}).  f is evaluated through the maximisation form of Prop. 2 at its maximiser
 * y: f = <y, theta> - (lambda / p) sum_i y_i^p, summed in float64 together with the multiplier
 * term - gamma (sum_i y_i - k), which is zero at the maximiser and keeps the rounding of the
 * float32 mask out of the value in first order.
 *   theta, target [rows][n] in (target: usually a 0/1 encoding of the wanted classes),
 *   loss_out [rows] out, grad_out [rows][n] out (required: beyond 2048 elements per row it also
 *   carries the mask between the two kernels; shorter rows take one kernel).
 *   Same shape rules, p values, workspace needs and errors as topk_mask_fwd.
 */
int topk_mask_loss(const float* theta, const float* target, int64_t rows, int64_t n, int64_t k,
                   double p, double lambda, float* loss_out, float* grad_out, void* stream);

/*
 * The sorting permutation itself (Sec. 3, argsort): perm_out[r][i] = original index of the i-th
 * largest value of row r (0-based), ties by ascending index, -0 equal to +0.  For rows of up to
 * TOPK_SHORT_ROW_MAX elements this is the permutation the operators above build in registers.
 * Longer rows are sorted completely here (segmented radix sort through the workspace of
 * TOPK_OP_ARGSORT), whereas the operators only order the part of such a row that can pool (the
 * elements inside a value window around positions k and k+1, in this same order); their outputs
 * do not depend on the order of the rest.
 */
int topk_argsort_desc(const float* theta, int64_t rows, int64_t n, int32_t* perm_out, void* stream);

/*
 * Scratch memory (bytes) that `op` (a TOPK_OP_* code) needs for this shape with the routes that
 * are set when it is called (topk_set_route; ask again after changing them); for the first five
 * codes 0 when rows fit one wavefront (n <= TOPK_SHORT_ROW_MAX; n <= 2048 for the dense
 * operators other than top-k in magnitude with p = 4/3).  Returns 0 for invalid arguments as
 * well.
 */
size_t topk_workspace_bytes(int op, int64_t rows, int64_t n, int64_t k, double p);

/*
 * Register caller-owned device scratch memory (256-byte aligned) for later calls; the library
 * never frees it.  dev_ptr == NULL (with bytes == 0) unregisters.  Returns TOPK_OK or
 * TOPK_ERR_INVALID (misaligned pointer, or NULL with bytes != 0).
 */
int topk_set_workspace(void* dev_ptr, size_t bytes);

/*
 * Test and tuning control: chooses among code paths that compute the same results (the GPU tests
 * compare them bit for bit).  Process-wide, takes effect for later calls; not meant for production
 * callers, whose default is always TOPK_*_AUTO.
 *   TOPK_ROUTE_LONG_ROWS        how rows above TOPK_SHORT_ROW_MAX elements are handled:
 *                               TOPK_LONG_ROWS_AUTO (by shape), _SELECT (multi-launch candidate
 *                               selection, sorted (key, index) lists and scatter, for every such
 *                               row), _SORT (rows sorted completely), _WIDE (multi-launch
 *                               selection, key-only sort and outputs by value: what AUTO takes
 *                               for rows above 131072 elements), _ONE_LAUNCH_INDEXED (up to 131072
 *                               elements: the one-launch kernel that sorts (key, index) pairs,
 *                               which AUTO only takes up to 8192 elements)
 *   TOPK_ROUTE_SHORT_ROW_LANES  lanes of a wavefront that share a short row: 0 (by shape) or a
 *                               power of two up to 64 (clamped to what the row length allows)
 *   TOPK_ROUTE_SHORT_ROW_KERNEL for rows of up to 128 elements: TOPK_SHORT_ROW_KERNEL_AUTO (dense
 *                               outputs from the kernel that orders values only), _INDEXED (the
 *                               kernel that builds the permutation, as the compact output and
 *                               topk_argsort_desc always do), _GENERAL (the general short-row
 *                               kernel of rows up to TOPK_SHORT_ROW_MAX elements)
 *   TOPK_ROUTE_GENERAL_ROUNDS   topk_general_*: merging rounds after which a wavefront hands its rows
 *                               to the sequential block stack; 0 = the default, 1..4096
 * Returns TOPK_OK or TOPK_ERR_INVALID (unknown control or value).
 */
#define TOPK_ROUTE_LONG_ROWS 0
#define TOPK_ROUTE_SHORT_ROW_LANES 1
#define TOPK_ROUTE_SHORT_ROW_KERNEL 2
#define TOPK_ROUTE_GENERAL_ROUNDS 3
#define TOPK_LONG_ROWS_AUTO 0
#define TOPK_LONG_ROWS_SELECT 1
#define TOPK_LONG_ROWS_SORT 2
#define TOPK_LONG_ROWS_WIDE 3
#define TOPK_LONG_ROWS_ONE_LAUNCH_INDEXED 4
#define TOPK_SHORT_ROW_KERNEL_AUTO 0
#define TOPK_SHORT_ROW_KERNEL_INDEXED 1
#define TOPK_SHORT_ROW_KERNEL_GENERAL 2
int topk_set_route(int which, int value);

/* Static, human-readable text for a return code. */
const char* topk_strerror(int code);

#ifdef __cplusplus
}
#endif
#endif /* SPARSE_TOPK_H_ */
