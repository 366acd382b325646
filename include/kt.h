/*
 * kt.h -- C ABI of the MI355X (gfx950) KurTail rotation-learning library.
 *
 * The library covers the data-parallel hot path of KurTail (arXiv 2503.01483,
 * "Learning the Rotations" / "Optimization in the Orthogonal Space"): rotate the
 * stored block-input activations X by an orthogonal R, reduce every token row of
 * Y = X R to its kurtosis (Background, "Kurtosis", Eq. 3), average into the loss,
 * back-propagate to dL/dR = X^T (dL/dY), and retract R onto the orthogonal group
 * with a Cayley step; plus the per-token symmetric int4 fake quantiser used to
 * check the rotated activations (Background, "Uniform Quantization for k-bit
 * Precision"; Setup).  Further entry points cover the optimiser and the loss exactly as
 * the paper names them (Cayley Adam, pooled kurtosis after an RMSNorm), the quantities the
 * paper evaluates rotations with, and the application of rotations (Hadamard rows, fusion
 * into weights).
 *
 * Conventions common to every entry point
 *  - All data pointers are DEVICE pointers on the current HIP device unless the
 *    comment says "host".  The caller owns every buffer; the library allocates,
 *    frees and retains nothing, and keeps no state between calls.
 *  - Work is enqueued on `stream` (a hipStream_t passed as void*; NULL = the
 *    default stream).  No call synchronises with the host; scalar results stay
 *    on the device.
 *  - Argument errors are reported synchronously (nothing is enqueued, nothing is
 *    written) through the return value; kt_last_error() gives the text.
 *    Faults on the device surface at the caller's next synchronisation.
 *  - Inputs and outputs must not overlap, except the in/out arguments (R, M, v of the
 *    Cayley steps) and Y == X in kt_hadamard_rows.
 *  - `batch` independent problems are laid out back to back: problem b of X
 *    starts at X + b*n*ldx elements, of R at R + b*d*ldr, of dR at dR + b*d*d.
 *  - Results are deterministic: the same inputs give bitwise the same outputs
 *    (fixed-order reductions, no floating-point atomics).
 *  - `workspace` is device scratch of at least kt_workspace_bytes(...) bytes,
 *    256-byte aligned; its contents are undefined before and after a call.
 */
#ifndef KT_H_
#define KT_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef int32_t kt_status;
enum {
  KT_OK = 0,
  KT_ERR_INVALID_ARG = 1,         /* null pointer, non-positive size, bad scalar   */
  KT_ERR_BAD_SHAPE = 2,           /* d not a multiple of 128, ld too small/unaligned */
  KT_ERR_BAD_DTYPE = 3,           /* unsupported dtype combination                  */
  KT_ERR_WORKSPACE_TOO_SMALL = 4,
  KT_ERR_DEVICE = 5,              /* the HIP runtime refused a launch               */
  KT_ERR_NOT_SUPPORTED = 6
};

/* Element types and operation codes travel as plain 32-bit integers (like kt_status): a value outside
 * the lists below is an argument error the library reports, never an invalid enumeration value. */
typedef int32_t kt_dtype;
enum { KT_F32 = 0, KT_BF16 = 1 };
typedef int32_t kt_op;
enum { KT_OP_LOSS_GRAD = 0, KT_OP_CAYLEY = 1, KT_OP_FAKEQUANT = 2, KT_OP_POOLED_LOSS_GRAD = 3,
       KT_OP_QUANT_METRICS = 4, KT_OP_FUSE_ROTATION = 5,
       KT_OP_SENSITIVITY = 6, KT_OP_LOSS_GRAD_RECOMPUTE = 7,
       KT_OP_POOLED_LOSS_GRAD_RECOMPUTE = 8 };

/* Library version (major*10000 + minor*100 + patch). Host call. */
int32_t kt_version(void);

/* Identifier of the source files this binary was compiled from (set by the build script; the Python
 * binding compares it with the sources it sees and rebuilds a library that no longer matches).
 * Static storage.  Host call. */
const char* kt_build_id(void);

/* Text of the last error raised on the calling host thread ("" if none).
 * Points to thread-local static storage; never free it. */
const char* kt_last_error(void);

/* Scratch bytes the given operation needs for these sizes (0 on bad sizes).
 * For KT_OP_CAYLEY `n` is ignored.  KT_OP_LOSS_GRAD / KT_OP_POOLED_LOSS_GRAD: the recommended size
 * (with room to keep Y, see kt_kurtosis_loss_grad); KT_OP_LOSS_GRAD_RECOMPUTE /
 * KT_OP_POOLED_LOSS_GRAD_RECOMPUTE: the least those entry points accept.  Host call, launches nothing. */
size_t kt_workspace_bytes(kt_op op, int64_t batch, int64_t n, int64_t d, kt_dtype x_dtype);

/*
 * Kurtosis loss and its Euclidean gradient with respect to R.
 *
 *   Y = X R                                   ("Learning the Rotations": linear layer)
 *   per token row i:  mu_i = mean_j y_ij, c = y - mu, m_k = mean_j c^k,
 *                     kappa_i = m4 / m2^2     (Eq. 3; population moments, not excess)
 *   loss = (1/n) sum_i f(kappa_i),  f(k) = k            if kappa_target == 0
 *                                   f(k) = |k - target| otherwise   (kurtosis loss,
 *                                   per-token-row reading; target 9/5 = uniform)
 *   dL/dy_ij = s_i 4/(n d m2_i^2) [c_ij^3 - m3_i - kappa_i m2_i c_ij],  s_i = f'(kappa_i)
 *   dR = X^T (dL/dY)
 *
 * Y is consumed in the forward GEMM's epilogue (row moments).  For the backward pass it is either
 * KEPT by that epilogue (fp32, token-minor, 4 n d bytes of workspace per problem) and dL/dY computed
 * from it entry by entry, or RECOMPUTED by a second GEMM whose epilogue forms dL/dY: the first when
 * the workspace handed in has the room (kt_workspace_bytes(KT_OP_LOSS_GRAD) asks for it while Y is at
 * most 64 GiB), the second otherwise (KT_OP_LOSS_GRAD_RECOMPUTE is the smaller size).  Both give the
 * same bits: dL/dY comes from the same fp32 accumulators through the same arithmetic.  dL/dY exists
 * only as the token-minor scratch operand of the last GEMM (which reads X itself in place when X is
 * bf16 and d a multiple of 256, through a token-minor copy otherwise).
 *
 *  X        [batch][n][ldx] row-major, x_dtype (KT_BF16, or KT_F32 for the fp32 path);
 *           d <= ldx <= 2^22, rows 16-byte aligned (ldx % 8 == 0 for bf16, % 4 for fp32).
 *  R        [batch][d][ldr] row-major, r_dtype.  With bf16 X, R may be the fp32 master
 *           (rounded to bf16, nearest-even, inside) or already bf16; the loss and
 *           gradient are those at the bf16-rounded R.  With fp32 X, R must be fp32.
 *  d        multiple of 128, <= 16384.   1 <= n <= 2^22, any value (tail rows are masked).
 *  loss     [batch] fp32, written.
 *  row_kurt [batch][n] fp32 or NULL.
 *  dR       [batch][d][d] fp32 or NULL (NULL: loss only, the backward GEMMs are skipped).
 *  A row without spread (m2 <= 1e-10 of its mean square: sigma below 1e-5 of the mean, which fp32
 *  products cannot resolve) counts with kappa = 0 and contributes no gradient.  Above that the row
 *  values carry an error of about 1e-6 |mean| / sigma on top of the path tolerance.
 */
kt_status kt_kurtosis_loss_grad(const void* X, int64_t ldx, const void* R, int64_t ldr,
                                int64_t batch, int64_t n, int64_t d,
                                kt_dtype x_dtype, kt_dtype r_dtype, float kappa_target,
                                float* loss, float* row_kurt, float* dR,
                                void* workspace, size_t workspace_bytes, void* stream);

/*
 * The loss exactly as the paper writes it (loss equation of the "Kurtosis" paragraph) on the
 * small network of "Learning the Rotations" (linear layer R followed by an RMSNorm without
 * gain): with Y = X R, rho_i = sqrt(mean_j y_ij^2 + rms_eps), Z = Y / rho,
 *
 *   kappa = kurtosis (Eq. 3) of ALL n*d entries of Z taken as one sample
 *           (the concatenation of the activations of all tokens),
 *   loss  = |kappa - kappa_target|   (kappa_target = 1.8, the uniform distribution, in the
 *           paper; kappa_target == 0 gives loss = kappa),
 *
 * per problem of the batch (the paper's 1/L sum over layers is the mean of `loss` over the
 * batch).  dR = dloss/dR with R a free matrix, including the Jacobian of the RMSNorm.
 * Arguments as for kt_kurtosis_loss_grad; `kappa` [batch] fp32 or NULL receives kappa.
 * Three passes over X (moments, recompute + dL/dY, X^T G) for every d, d = 128 included:
 * the gradient needs the pooled statistics of the whole problem first.
 * Workspace: kt_workspace_bytes(KT_OP_POOLED_LOSS_GRAD, ...) (Y kept) or (KT_OP_POOLED_LOSS_GRAD_RECOMPUTE, ...).
 */
kt_status kt_pooled_kurtosis_loss_grad(const void* X, int64_t ldx, const void* R, int64_t ldr,
                                       int64_t batch, int64_t n, int64_t d,
                                       kt_dtype x_dtype, kt_dtype r_dtype, float kappa_target,
                                       float rms_eps, float* loss, float* kappa, float* dR,
                                       void* workspace, size_t workspace_bytes, void* stream);

/*
 * One Cayley SGD step on the orthogonal group ("Optimization in the Orthogonal
 * Space"; the paper names the optimiser and defers the formula to its reference):
 *
 *   A  = dR R^T - R dR^T          (skew-symmetric)
 *   R+ = (I + lr/2 A)^-1 (I - lr/2 A) R
 *
 * The solve is the fixed-point iteration Z <- R - (lr/2) A (R + Z), run on the
 * device until the iterate is within the resolution of the arithmetic of its limit.  The
 * iteration is linear, so the changes d_k = max |Z_k - Z_k-1| shrink geometrically with a ratio
 * rho that is estimated from them (over two steps, d_k / d_k-2 = rho^2, once three are there: the
 * even and odd terms of the series can have different patterns), and the iterate is accepted
 * when four times the bound d_k rho / (1 - rho) on its distance to the limit is below 3e-7, or
 * when the changes are small (<= 2e-5) and have stopped shrinking (the rounding floor).  It
 * contracts when (lr/2)||A||_2 < 1 and the library enqueues at most 32 iterations (enough up to
 * about 0.55).  No learning-rate
 * clamp is applied: the caller chooses lr.  For d >= 1024 the d^3 products run on the
 * bf16 matrix cores as three-term bf16 products (about 2^-17 relative per term).
 *
 *  R        [batch][d][d] fp32, in/out (master copy).  d multiple of 128, <= 16384.
 *  dR       [batch][d][d] fp32.  R and dR 16-byte aligned.
 *  R_lowp   [batch][d][d] bf16 copy of the new R (nearest-even), or NULL.
 *  ortho_err[batch] fp32: max_ij |(R+^T R+ - I)_ij| of the result, or NULL (skips one GEMM).
 *  info     [batch] int32: number of iterations used, or -1 if the iteration did not
 *           converge within the library's limit, or NULL.  A step that did not converge is
 *           rejected: R comes back unchanged, R_lowp is the bf16 copy of that unchanged R, and
 *           ortho_err is unspecified.
 */
kt_status kt_cayley_step(float* R, const float* dR, void* R_lowp, int64_t batch, int64_t d,
                         float lr, float* ortho_err, int32_t* info,
                         void* workspace, size_t workspace_bytes, void* stream);

/*
 * kt_cayley_step for callers that cannot allocate device memory and hold no workspace: code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, checks,
 * kernels and results as kt_cayley_step, but the scratch is a static device array inside the library
 * image (8 MiB per GPU the library runs on, held until the process ends); the call allocates and frees
 * nothing (its address is looked up with hipGetSymbolAddress once per device, at the first call with
 * that device current).
 *  Limit: kt_workspace_bytes(KT_OP_CAYLEY, batch, 0, d, KT_F32) <= 8 MiB, i.e. d = 512 with batch 1,
 *  d = 384 with batch <= 2, d = 256 with batch <= 6, d = 128 with batch <= 25; anything larger returns
 *  KT_ERR_NOT_SUPPORTED before anything is enqueued.
 *  All calls on one GPU share that GPU's array: calls that overlap in time on one GPU (different
 *  streams, different host threads) race and must be serialised by the caller.  The array keeps the
 *  previous call's contents; every counter the kernels need at zero is cleared by a fill kernel at the
 *  start of each call.
 */
kt_status kt_cayley_step_static(float* R, const float* dR, void* R_lowp, int64_t batch, int64_t d,
                                float lr, float* ortho_err, int32_t* info, void* stream);

/*
 * One Cayley Adam step on the orthogonal group: the optimiser the paper uses for all
 * rotations ("Learning the Rotations"; Setup).  The paper prints no formula and defers to
 * the cited work on optimisation over the Stiefel manifold; the step implemented here is
 * that algorithm specialised to square orthogonal R, with the Cayley transform iterated to
 * convergence instead of a fixed number of inner iterations (step counter k = `step` >= 1):
 *
 *   M  <- beta1 M + (1 - beta1) dR                      first moment
 *   v  <- beta2 v + (1 - beta2) ||dR||_F^2              scalar second moment
 *   r   = (1 - beta1^k) sqrt(v / (1 - beta2^k) + eps)
 *   W   = (M R^T - R M^T) / (2 r)                       skew-symmetric
 *   M  <- r W R                                         momentum moved into the tangent space at R
 *   a   = min(lr, 2 q / (||W||_F + eps))                keeps the iteration below contractive
 *   R+  = (I + a/2 W)^-1 (I - a/2 W) R                  fixed point Z <- R - (a/2) W (R + Z)
 *
 *  R        [batch][d][d] fp32, in/out.  d multiple of 128, <= 16384.
 *  dR       [batch][d][d] fp32.  R, dR and M 16-byte aligned.
 *  M        [batch][d][d] fp32 momentum, in/out (zeros before the first step).
 *  v        [batch] fp32 second moment, in/out (1 before the first step).
 *  R_lowp, ortho_err, info: as for kt_cayley_step.
 *  scalars  [batch][3] fp32 {r, a, ||W||_F} of this step, or NULL.
 *  Workspace: kt_workspace_bytes(KT_OP_CAYLEY, ...).  A zero gradient with zero momentum
 *  gives W = 0 and leaves R unchanged.
 */
kt_status kt_cayley_adam_step(float* R, const float* dR, float* M, float* v, int64_t step,
                              void* R_lowp, int64_t batch, int64_t d, float lr, float beta1,
                              float beta2, float eps, float q, float* ortho_err, int32_t* info,
                              float* scalars, void* workspace, size_t workspace_bytes, void* stream);

/*
 * Rotate and fake-quantise to symmetric int4, one scale per token row
 * (Background, "Uniform Quantization for k-bit Precision" with k = 4, b = 0;
 * Setup: per-token dynamic symmetric quantisation; error as in Eq. 1):
 *
 *   y = x R (fp32 accumulation);  s_i = (clip_ratio * max_j |y_ij|) / 7   (or scales_in)
 *   q_ij = clamp(rint(y_ij * (1/s_i)), -7, 7)   (fp32, round half to even)
 *   err_i = { sum_j (y_ij - q_ij s_i)^2, sum_j y_ij^2 }
 *
 *  X, R, batch, n, d, dtypes: as for kt_kurtosis_loss_grad.
 *  clip_ratio in (0, 1]; 1 is the plain symmetric scale.
 *  scales_in  [batch][n] fp32 or NULL; if given it is used verbatim.
 *  scales_out [batch][n] fp32 or NULL.
 *  codes      [batch][n][d] int8, one code per byte in [-7, 7], 16-byte aligned, or NULL.
 *  err        [batch][n][2] fp32 or NULL.
 *  A row with scale 0 gets codes 0.
 *  Workspace: kt_workspace_bytes(KT_OP_FAKEQUANT, ...).  It holds an fp32 staging buffer of at most
 *  1 GiB: when the scales are computed here, y is rotated once, a slice of token rows at a time,
 *  and a row kernel takes the maximum and quantises the staged values (one GEMM pass instead of a
 *  second one that recomputes y).  With scales_in the codes come straight out of the GEMM's registers.
 *  d = 128 in bf16 is a single fused pass with no staging.
 */
kt_status kt_rotate_fakequant_int4(const void* X, int64_t ldx, const void* R, int64_t ldr,
                                   int64_t batch, int64_t n, int64_t d,
                                   kt_dtype x_dtype, kt_dtype r_dtype, float clip_ratio,
                                   const float* scales_in, float* scales_out, int8_t* codes,
                                   float* err, void* workspace, size_t workspace_bytes,
                                   void* stream);

/*
 * Per-token quantisation-quality figures of the rotated activations Y = X R, the quantities
 * the paper evaluates a rotation with:
 *   amax      [batch][n][2] fp32 {max_j |x_ij|, max_j |y_ij|};  success[batch] int64 = number of
 *             tokens whose largest magnitude shrank ("Evaluation ... on Channel Outliers": the
 *             success rate is success / n)
 *   threshold [batch][n] fp32: the `quantile` quantile of |y_i| over the row (linear interpolation
 *             between order statistics; quantile = 1: the maximum).  Setup appendix: 0.98.
 *   err_sym   [batch][n][2] fp32 {sum_j (y - yhat)^2, sum_j y^2}, symmetric int4 with
 *             s = threshold / 7, values beyond the threshold clipped (Background, "Uniform
 *             Quantization for k-bit Precision", b = 0; Setup: per-token, clipped at a quantile)
 *   err_asym  [batch][n][2] fp32, asymmetric int4: b = min_j y, s = (max_j y - b) / 15
 *             (Background; Setup: KV caches)
 *   Y         [batch][n][d] fp32: receives the rotated activations, or NULL (then they live in
 *             the workspace).  Every output pointer may be NULL.
 * Y is materialised (this is an evaluation tool, not the training step): one GEMM pass, then one
 * wave per token with the row in registers (radix select on the bit patterns for the quantile).
 * d <= 8192.
 * Workspace: kt_workspace_bytes(KT_OP_QUANT_METRICS, ...) (sized for Y == NULL: the rotated rows then
 * pass through an fp32 staging slice of at most 1 GiB, a few problems or token rows at a time).
 */
kt_status kt_rotate_quant_metrics(const void* X, int64_t ldx, const void* R, int64_t ldr,
                                  int64_t batch, int64_t n, int64_t d,
                                  kt_dtype x_dtype, kt_dtype r_dtype, float quantile,
                                  float* Y, float* amax, float* threshold, float* err_sym,
                                  float* err_asym, int64_t* success,
                                  void* workspace, size_t workspace_bytes, void* stream);

/*
 * Quantisation sensitivity of a tensor (Background: Definition "Quantization Sensitivity" and
 * Eq. 1): for the symmetric `bits`-bit uniform quantiser q = clamp(rint(y / s), -L, L) s,
 * L = 2^(bits-1) - 1, over ALL `count` entries of Y as one sample,
 *   out[0] = s_opt, the step minimising MSE(s) (three stages of a 32-point grid: s_max 2^(-j/4)
 *            with s_max = max|y| / L, then twice 32 points between the neighbours of the best),
 *   out[1] = MSE(s_opt),   gamma[i] = | MSE(s_opt (1 + alphas[i])) - MSE(s_opt) |.
 *  Y       device fp32 [count] (e.g. the Y output of kt_rotate_quant_metrics).
 *  alphas  device fp32 [n_alpha], n_alpha <= 31 (fractions of the optimal step, may be negative);
 *  out [2], gamma [n_alpha]: device fp32.  The search runs on the device; no host sync.
 * Workspace: kt_workspace_bytes(KT_OP_SENSITIVITY, 1, 1, 128, KT_F32).
 */
kt_status kt_quant_sensitivity(const float* Y, int64_t count, int32_t bits, const float* alphas,
                               int32_t n_alpha, float* out, float* gamma,
                               void* workspace, size_t workspace_bytes, void* stream);

/*
 * The online rotations of "Placement of the Rotations" (R3, R4, R5: random Hadamard matrices
 * applied to activations at run time):  Y[i][:] = (X[i][:] * signs) H_d / sqrt(d) for every
 * token row.  The paper does not say which Hadamard matrix of order d is meant (any one is a
 * rotation after scaling); this library uses, for d = r 2^t with r odd,
 *   H_d = H_m (x) S_{2^k}   (Kronecker product: element a 2^k + b of a row, a < m, b < 2^k),
 *   S the Sylvester matrix (S_1 = [1], S_2j = [[S_j, S_j], [S_j, -S_j]]),
 *   r = 1: m = 1 for t <= 12, else m = max(4, 2^(t-12)) and H_m = S_m  (H_d = S_d either way);
 *   r > 1: m = r 2^j for the smallest j >= 2 with m - 1 prime (Paley's first construction:
 *          H_m = I + [[0, 1^T], [-1, Q]], Q[u][v] = the quadratic character of u - v modulo
 *          q = m - 1), else with q = m/2 - 1 prime, q = 1 mod 4 (Paley's second construction:
 *          C = [[0, 1^T], [1, Q]], H_m = [[C + I, C - I], [C - I, -C - I]]).
 * This covers the hidden and FFN sizes 2^k, 3, 5, 7, 9, 11, 15, 27 x 2^k (5120, 6144, 13824,
 * 14336, 28672, ...); 11008 = 43 x 2^8 has no such factor up to order 128 and is refused.
 *  X, Y   [n][ldx], [n][ldy] row-major, `dtype` (KT_BF16: fp32 arithmetic, rounded to nearest
 *         even at the end; for m > 1 the result of the S factor passes through Y in bf16 before the
 *         H_m factor is applied); Y may be X (in place).  Rows 16-byte aligned.
 *  signs  [d] int8 +-1 (the random diagonal of a "random Hadamard" rotation), or NULL.
 *  d      as above with 128 <= 2^k <= 4096 and m <= 128.  For m = 1 without signs the transform
 *         is its own inverse.
 * No workspace.  HBM-bound: one read and one write of the rows per factor.
 */
kt_status kt_hadamard_rows(const void* X, int64_t ldx, void* Y, int64_t ldy, const int8_t* signs,
                           int64_t n, int64_t d, kt_dtype dtype, void* stream);

/*
 * Merging a fusible rotation (R1, R2 of "Placement of the Rotations") into a weight matrix, in
 * fp32:
 *   side 0:  Wout [k][d] = W [k][d] R          (the rotation on the right of a weight that writes
 *                                               the rotated stream: embedding, W_o, W_down, W_v)
 *   side 1:  Wout [d][k] = R^T W [d][k]        (its inverse on the left of a weight that reads it:
 *                                               W_q, W_k, W_v, W_up, W_gate; W_o for R2)
 * with x W for row-vector activations x.  W, R, Wout fp32 row-major with leading dimensions ldw,
 * ldr, ldo (multiples of 4); d multiple of 128; Wout must not overlap W.
 * Workspace: kt_workspace_bytes(KT_OP_FUSE_ROTATION, 1, k, d, KT_F32)  (n = k).
 */
kt_status kt_fuse_rotation(const float* W, int64_t ldw, const float* R, int64_t ldr, float* Wout,
                           int64_t ldo, int64_t k, int64_t d, int32_t side,
                           void* workspace, size_t workspace_bytes, void* stream);

/*
 * Measurement aid (not part of the method; off by default).  When enabled, the
 * library brackets its large launches with HIP events on the caller's stream so a
 * benchmark can read per-kernel durations without a profiler attached.  This is the
 * only process-global state the library has; enable/disable/read are host calls and
 * must not run concurrently with other library calls.
 *   kernel ids: 0 forward GEMM + row moments, 1 backward recompute GEMM + dL/dY,
 *               2 gradient GEMM X^T G, 3 token-minor copy of X (fp32, or d not a multiple of 256: bf16 with
 *               d % 256 == 0 reads X as it is),
 *               4 every launch of kt_cayley_step, 5 every launch of kt_rotate_fakequant_int4
 * kt_profile_enable(max_records): records up to max_records bracketed launches (0 turns
 *   profiling off and releases the events).
 * kt_profile_read(id, &total_ms, &launches): waits for the recorded events of that id and
 *   returns their summed duration and count; kt_profile_reset() forgets all records.
 */
kt_status kt_profile_enable(int32_t max_records);
kt_status kt_profile_read(int32_t kernel_id, double* total_ms, int32_t* launches);
kt_status kt_profile_reset(void);

#ifdef __cplusplus
}
#endif
#endif /* KT_H_ */
