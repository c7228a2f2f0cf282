/*
 * dartqr.h -- C ABI of the MI355X (gfx950) QR-Orth calibration-step library.
 *
 * One QR-Orth step is the loop body of Alg. 1 (Sec. 4.3) of DartQuant (arXiv 2511.04063):
 *     R <- qr(Z);   O <- X @ R;   L <- Whip(O);   Z <- Z - eta * dL/dZ
 * with Whip(x) = sum_i exp(-|x_i|) (Eq. 4, Sec. 4.2).  The paper names the ORTHOGONAL
 * factor R and the UPPER-TRIANGULAR factor U (Z = R U, Sec. 4.3); so does this header.
 *
 * Conventions shared by every entry point
 *  - All matrix pointers are DEVICE pointers (HIP device memory of the context's device),
 *    row-major, leading dimensions ("ld*") counted in ELEMENTS.  Scalars are host values.
 *  - fp32 matrices: base pointer 16-byte aligned, ld a multiple of 4 and >= the row length.
 *    bf16 matrices: base pointer 16-byte aligned, ld a multiple of 8 and >= the row length.
 *    Violations return DQ_ERR_ALIGN / DQ_ERR_SHAPE; there is no silent slow path.
 *  - Sizes: 1 <= n <= DQ_MAX_N, T >= 1, b >= 0 (b == 0 is a no-op returning DQ_OK).  n and T
 *    need not be multiples of anything.
 *  - Batches: problem i of a batch of b lives at  base + i * rows * ld  (its rows follow
 *    the previous problem's rows); per-problem scalars (loss) at index i.
 *  - Ownership: the library never allocates or frees device memory.  The caller owns every
 *    buffer, including the workspace, and keeps it alive until the stream has passed the
 *    call.  Inputs are read-only unless stated; outputs must not alias inputs.
 *  - Asynchrony: compute calls only enqueue work on the context's stream and return; results
 *    (including device scalars) are valid in stream order.  Only dq_device_flags and
 *    dq_profile_read synchronise.
 *  - Errors: arguments are checked on the host before anything is enqueued; a non-DQ_OK
 *    return means nothing was launched and no output was touched.  Numerical trouble
 *    (singular Z, non-finite values) sets bits in a device status word (dq_device_flags);
 *    outputs are then unspecified but every kernel still terminates normally.
 *  - One context per stream; a context is not re-entrant.  Calls on one context are
 *    serialised by its stream and share its workspace.
 */
#ifndef DARTQR_H
#define DARTQR_H

#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

#define DQ_MAX_N 8192          /* largest rotation size the panel factorisation supports */

typedef struct dq_ctx dq_ctx;  /* opaque; bound to one device and one HIP stream */

typedef enum {
    DQ_OK = 0,
    DQ_ERR_NULL = 1,           /* a required pointer is null                                  */
    DQ_ERR_SHAPE = 2,          /* a size is out of range or a leading dimension too small     */
    DQ_ERR_DTYPE = 3,          /* unknown dq_dtype / dq_reduce value                          */
    DQ_ERR_ALIGN = 4,          /* pointer or leading-dimension alignment rule violated         */
    DQ_ERR_WORKSPACE = 5,      /* no workspace set, or it is smaller than dq_workspace_bytes  */
    DQ_ERR_HIP = 6,            /* a HIP runtime call failed (launch, event)                   */
    DQ_ERR_UNSUPPORTED = 7     /* valid request outside the implemented range (n > DQ_MAX_N)  */
} dq_status;

typedef enum { DQ_F32 = 0, DQ_BF16 = 1 } dq_dtype;

/* How Whip (Eq. 4, defined for one activation vector) is reduced over the T token rows of a
 * block (the loss step of Alg. 1 leaves this open): mean over tokens of the per-token sum, or the sum. */
typedef enum { DQ_REDUCE_TOKEN_MEAN = 0, DQ_REDUCE_SUM = 1 } dq_reduce;

/* The objective S4 evaluates on the rotated block.  DQ_OBJ_WHIP is the paper's (Eq. 4).  The other three are the
 * alternatives it compares against (Sec. 4.1; Sec. 5, ablation of the optimisation objective), named there without
 * formulas; per token row y of n channels, with mu the row mean, d = y - mu and m_k = (1/n) sum_i d_i^k:
 *   DQ_OBJ_VARIANCE  m2
 *   DQ_OBJ_KURTOSIS  m4 / m2^2  (a constant row counts 0)
 *   DQ_OBJ_QUANT     (1/n) sum_i (y_i - yhat_i)^2 for the per-token asymmetric uniform quantiser of Sec. 5:
 *                    lo = min y, hi = max y, delta = (hi - lo) / (2^bits - 1), q_i = the nearest level to (y_i - lo) / delta
 *                    (decided in fp32), yhat_i = lo + delta q_i; the derivative holds the codes fixed and sends the
 *                    dependence on lo / hi to the first position of the minimum / maximum (a constant row counts 0)
 * Rows are combined like Eq. 4 (dq_reduce).  These three need n <= DQ_MAX_N. */
typedef enum { DQ_OBJ_WHIP = 0, DQ_OBJ_VARIANCE = 1, DQ_OBJ_KURTOSIS = 2, DQ_OBJ_QUANT = 3 } dq_objective;

/* bits of the device status word */
#define DQ_FLAG_SINGULAR   1u   /* a zero appeared on diag(U): Z is singular (dZ undefined)  */
#define DQ_FLAG_NONFINITE  2u   /* a NaN or Inf was seen in a pivot or in the loss           */
#define DQ_FLAG_ILLCOND_PANEL 4u /* informational: a tall 64-column panel of the QR was too ill-conditioned for the
                                   many-CU panel route and was factored by the one-workgroup Householder kernel
                                   instead; results are valid */
#define DQ_FLAG_BAD_INDEX  8u   /* dq_gather_rows met an index outside [0, T_all): that row was not written  */
#define DQ_FLAG_SYNC_TIMEOUT 16u /* a device-side wait between the library's streams (DQ_OPT_DEVICE_SYNC) ran into its
                                   time limit: the results of that call are invalid */

/* ---- context and workspace ---------------------------------------------------------- */

/* Create a context on the current HIP device for `hip_stream` (a hipStream_t, may be null for
 * the default stream).  *out receives the context.  Allocates host memory and HIP events only. */
dq_status dq_create(dq_ctx** out, void* hip_stream);
dq_status dq_destroy(dq_ctx* ctx);

/* Bytes of device workspace that any call with these sizes needs (a host computation).
 * x_dtype is the storage type of X.  *out receives the size.  Problems of a batch run one after
 * another and share the workspace, except for n == 128 (per-head rotations): there all b problems
 * run in the same kernel launches and the size grows with b (7 matrices of 64 KiB and
 * ceil(T/2048) partial gradients per problem).  A batch gives the same bits as its problems
 * run one by one. */
dq_status dq_workspace_bytes(int b, int n, int T, dq_dtype x_dtype, size_t* out);

/* Hand the context a caller-owned device buffer (256-byte aligned).  Enqueues one small kernel
 * that clears the status word at its start.  May be called again with another buffer. */
dq_status dq_set_workspace(dq_ctx* ctx, void* dptr, size_t bytes);

const char* dq_status_string(dq_status s);

/* Settings of a context that choose between implementations of the same result (A/B measurements, tests that must
 * reach a particular route).  Results are the same up to rounding under every setting; defaults are the measured
 * best.  Takes effect for the calls that follow.  DQ_ERR_DTYPE for an unknown option, DQ_ERR_SHAPE for a value out of
 * range; the setting is unchanged on error. */
typedef enum {
    DQ_OPT_ACCUM_PANELS = 0,        /* panels whose reflectors are merged before they are applied to the accumulated
                                       rotation: 1, 2 or 4; 0 (default): by size, 2 below n = 8192 and 4 from there on */
    DQ_OPT_TALL_PANEL_MIN_ROWS = 1, /* 64-column panels at least this tall take the many-compute-unit route
                                       (CholeskyQR2 + Householder reconstruction); 0: never, default 64 */
    DQ_OPT_SINGLE_STREAM = 2,       /* non-zero: every piece of the QR on the context's stream, no overlap (default 0) */
    DQ_OPT_FUSED_WHIP = 3,          /* zero: Eq. 4 always as a pass of its own, never in the epilogue of X @ R (default 1) */
    DQ_OPT_HEADS_BATCHED = 4,       /* zero: 128 x 128 problems take the general route one by one (default 1) */
    DQ_OPT_DEVICE_SYNC = 5,         /* how the pieces of the QR on the library's streams wait for each other.  0: HIP
                                       events.  1 (default): through a word in device memory that the producing stream
                                       sets and the consuming stream polls (a cross-stream wait on an event that is still
                                       pending costs the host 10-20 us here, several per panel), IF a probe at the first
                                       call on a stream shows that the streams involved make progress independently
                                       (they do unless they share a hardware queue); otherwise events.  Every poll is
                                       bounded (DQ_FLAG_SYNC_TIMEOUT). */
    DQ_OPT_SPLIT_GEMM = 6,          /* the n x n x n fp32 products of S6 (R^T G and R M) on the bf16 matrix cores from
                                       three-plane bf16 splits of both operands (x = x1 + x2 + x3 carries 24 mantissa
                                       bits; the six plane pairs above fp32 rounding are accumulated in fp32).  0: never
                                       (fp32 matrix cores); 1 (default): when n is a multiple of 256 and at least 2560,
                                       where it is faster; 2: whenever n is a multiple of 256. */
    DQ_OPT_FUSED_PANEL = 7,         /* S1: a tall 64-column panel that follows a tall panel and is followed by one as ONE
                                       launch whose workgroups hand over to each other through words in device memory
                                       (bounded polls, DQ_FLAG_SYNC_TIMEOUT) instead of three dependent launches.  Only
                                       taken where DQ_OPT_DEVICE_SYNC's hand-over is in use (not under stream capture).
                                       0: never; 1 (default) and 2: wherever the panel qualifies. */
    DQ_OPT_TWO_LEVEL_ROWS = 8       /* S1: two-level blocking.  While a block of 256 columns (four panels) has more rows than
                                       this, its panels' reflectors are applied one by one only to the 320 columns after the
                                       block's start; everything further right gets ONE update per block with the block's
                                       merged reflector (reduction length 256 instead of 64: a quarter of the passes over the
                                       trailing matrix).  Needs DQ_OPT_DEVICE_SYNC's hand-over and n a multiple of 256.
                                       0: never; -1 (default): 2048 rows in matrices of order 6144 or more, never below. */
} dq_option;
dq_status dq_set_option(dq_ctx* ctx, dq_option option, int value);

/* The probe behind DQ_OPT_DEVICE_SYNC on two streams of the caller's choosing (hipStream_t, null = default stream):
 * enqueues a wait on `consumer_stream` that polls a word of the workspace for at most 2 ms, THEN a kernel on
 * `producer_stream` that sets the word, and waits on the host for both streams.  *usable = 1 if the wait saw the word,
 * 0 if it ran into its limit (the streams share a hardware queue, or are the same stream); the status word is not
 * touched.  Needs a workspace.  Host-synchronous; for diagnosis and tests. */
dq_status dq_stream_handover_probe(dq_ctx* ctx, void* consumer_stream, void* producer_stream, int* usable);

/* Waits for the stream, copies the device status word to *host_out and clears it on the device. */
dq_status dq_device_flags(dq_ctx* ctx, unsigned* host_out);

/* ---- the hot path ------------------------------------------------------------------- */

/* Sec. 4.3 / the QR step of Alg. 1:  Z (n x n) -> orthogonal R and, optionally, upper-triangular U with
 * Z = R U.  Computed by blocked Householder QR (Alg. 2 in blocked compact-WY form) followed by
 * sign normalisation so that diag(U) >= 0, which makes R unique for nonsingular Z.
 * Z: in, b x (n x n) fp32.  R: out, fp32.  U_or_null: out, fp32, strictly-lower part written as 0. */
dq_status dq_qr_orth(dq_ctx* ctx, int b, int n,
                     const float* Z, long ldz, float* R, long ldr,
                     float* U_or_null, long ldu);

/* Alg. 1, rotation and loss steps, and the chain rule to R:
 *   Y = X @ R;   loss = c * sum_t sum_i exp(-|Y_ti|)  (Eq. 4; c = 1/T or 1 per `red`);
 *   dY = -c * sgn(Y) * exp(-|Y|) with sgn(0) = 0;   G = X^T @ dY = dL/dR.
 * X: in, b x (T x n), dtype xdt (bf16 X is multiplied on the bf16 matrix cores against R rounded
 * to bf16, fp32 accumulate; fp32 X uses fp32 matrix cores).  R: in, fp32 (need not be orthogonal).
 * loss_dev: out, b device floats.  G: out, fp32 n x n.  Y_or_null: out, fp32 T x n, ldy.
 * dY_or_null: out, T x n in the dtype of X (bf16 or fp32), lddy. */
dq_status dq_rotate_loss_grad(dq_ctx* ctx, int b, int T, int n,
                              const void* X, dq_dtype xdt, long ldx,
                              const float* R, long ldr, dq_reduce red,
                              float* loss_dev, float* G, long ldg,
                              float* Y_or_null, long ldy, void* dY_or_null, long lddy);

/* The whole loop body of Alg. 1 with plain SGD:  Z is updated IN PLACE to
 * Z - lr * dL/dZ.  loss_dev (b device floats) and R_or_null receive the loss and the rotation of
 * the INPUT Z (before the update). */
dq_status dq_calib_step(dq_ctx* ctx, int b, int T, int n,
                        const void* X, dq_dtype xdt, long ldx,
                        float* Z, long ldz, float lr, dq_reduce red,
                        float* loss_dev, float* R_or_null, long ldr);

/* Alg. 1, the loop over mini-batches, with the calibration set in HOST memory: step k (k = 0 .. steps-1) is
 * dq_calib_step on batch k % num_batches, and batch k + 1 travels to the device on an internal stream while step k
 * runs (two staging slots).  One problem (b = 1).
 * X_host: HOST array of num_batches HOST pointers, each a T x n block of dtype xdt with leading dimension ldx.  Pinned
 *   buffers (hipHostMalloc) make the copies asynchronous; pageable ones work and serialise.  The blocks must stay
 *   valid and unchanged until the context's stream has finished the call's work.
 * staging_dev: DEVICE memory for two batches, 2 * T * ldx elements of xdt, 16-byte aligned; contents are overwritten.
 * Z: in/out, fp32 n x n.  losses_dev: out, `steps` DEVICE floats, the loss of each step's input Z.
 * The workspace is that of dq_workspace_bytes(1, n, T, xdt).  steps == 0 is a no-op. */
dq_status dq_calib_run_host_batches(dq_ctx* ctx, int T, int n,
                                    const void* const* X_host, int num_batches, dq_dtype xdt, long ldx,
                                    void* staging_dev, float* Z, long ldz, float lr, dq_reduce red,
                                    int steps, float* losses_dev);

/* ---- stages exported on their own (stage-level parity tests, reuse) -------------------- */

/* Eq. 4 and its derivative on an existing Y (fp32, T x n): loss_dev[i] and dY (dtype dydt). */
dq_status dq_whip_loss_grad(dq_ctx* ctx, int b, int T, int n,
                            const float* Y, long ldy, dq_reduce red,
                            float* loss_dev, void* dY, dq_dtype dydt, long lddy);

/* dq_whip_loss_grad for callers that cannot allocate device memory and have no workspace to hand over: code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Takes no context: hip_stream is the
 * hipStream_t to enqueue on (may be null).  The status word and the per-workgroup partial sums live in a fixed
 * array of device memory inside the library (256 + 8 * DQ_NOALLOC_MAX_BATCH bytes, one copy per GPU, held until the
 * process ends); the call allocates and frees nothing, creates no events, and enqueues kernels only (no memset
 * nodes).  Same arguments, results and argument errors as dq_whip_loss_grad; b > DQ_NOALLOC_MAX_BATCH returns
 * DQ_ERR_UNSUPPORTED (the array holds one partial sum per problem at least).  The status word is not readable: a
 * non-finite loss shows in loss_dev itself.  All calls on one GPU share the array, so calls that may overlap on one
 * GPU (different streams, different threads) race: serialise them. */
#define DQ_NOALLOC_MAX_BATCH 8192
dq_status dq_whip_loss_grad_noalloc(void* hip_stream, int b, int T, int n,
                                    const float* Y, long ldy, dq_reduce red,
                                    float* loss_dev, void* dY, dq_dtype dydt, long lddy);

/* The same stage for any dq_objective (Sec. 5, objective ablation): loss_dev[i] and dY = d loss / dY on an existing
 * Y (fp32, b blocks of T x n).  quant_bits (1..16) is read by DQ_OBJ_QUANT only.  DQ_OBJ_WHIP is dq_whip_loss_grad.
 * With the three row objectives dY may be null: then only loss_dev is written, e.g. the per-token quantisation error
 * of a rotated block as an evaluation metric (Sec. 5 measures activation quantisation error along the calibration). */
dq_status dq_objective_loss_grad(dq_ctx* ctx, dq_objective objective, int quant_bits, int b, int T, int n,
                                 const float* Y, long ldy, dq_reduce red,
                                 float* loss_dev, void* dY, dq_dtype dydt, long lddy);

/* Selects the objective that dq_rotate_loss_grad, dq_calib_step and dq_calib_step_adam evaluate from now on
 * (default DQ_OBJ_WHIP; Sec. 5, objective ablation).  With another objective Y and dY always pass through the
 * workspace (no fused epilogue, no batched 128-wide route).  DQ_ERR_DTYPE for an unknown objective, DQ_ERR_SHAPE for
 * quant_bits outside 1..16; the setting is unchanged on error. */
dq_status dq_set_objective(dq_ctx* ctx, dq_objective objective, int quant_bits);

/* The last step of Alg. 1, the derivative through Z = R U:  with B = R^T G and P = strict_lower(B - B^T),
 * dZ = R P U^{-T}.  R, U, G: in (U upper triangular, its strictly-lower part is not read).
 * dZ: out.  A zero on diag(U) sets DQ_FLAG_SINGULAR. */
dq_status dq_qr_backward(dq_ctx* ctx, int b, int n,
                         const float* R, long ldr, const float* U, long ldu,
                         const float* G, long ldg, float* dZ, long lddz);

/* The initial latent of the paper's runs (App., hyper-parameter settings: a randomised Hadamard matrix), read as
 * Z0_i = diag(s_i) H_n / sqrt(n) with H_n the Sylvester Hadamard matrix, H[r][c] = (-1)^popcount(r & c): an
 * orthogonal matrix for signs s = +-1.  n must be a power of two (DQ_ERR_UNSUPPORTED otherwise).  The random signs
 * are the caller's: signs_dev holds b*n DEVICE floats (row r of problem i is scaled by signs_dev[i*n + r]).
 * Z: out, b matrices. */
dq_status dq_hadamard_init(dq_ctx* ctx, int b, int n, const float* signs_dev, float* Z, long ldz);

/* Sec. 4.1, Eq. 1, the quantity the calibration drives down: counts_dev[i] = number of entries of the rotated block
 * Y_i (T x n fp32, b problems) with |y| > tau.  An evaluation metric, not part of the step.  counts_dev: b DEVICE
 * 64-bit unsigned integers (8-byte aligned), overwritten.  NaN entries are not counted. */
dq_status dq_outlier_count(dq_ctx* ctx, int b, int T, int n, const float* Y, long ldy, float tau,
                           unsigned long long* counts_dev);

/* Alg. 1, token sampling: X_out[i][t][:] = X_all[i][idx[i*T_out + t]][:] for t < T_out, b independent
 * problems (X_all: b blocks of T_all rows, X_out: b blocks of T_out rows, both with n columns of `dtype`).
 * Which tokens are kept (the paper samples 10 % of them at random) is the caller's choice: idx is a DEVICE array of
 * b*T_out int32 row numbers in [0, T_all), repeats allowed.  Rows must be 16-byte multiples and 16-byte aligned
 * (n a multiple of 8 for bf16, of 4 for fp32, with the usual leading-dimension rules).  An index out of range leaves
 * its output row untouched and raises DQ_FLAG_BAD_INDEX.  Needs a workspace only for the status word. */
dq_status dq_gather_rows(dq_ctx* ctx, int b, int T_all, int T_out, int n, const void* X_all, dq_dtype dtype,
                         long ldx_all, const int* idx, void* X_out, long ldx_out);

/* The last step of Alg. 1, the update alone:  Z <- Z - lr * dZ  (in place on Z). */
dq_status dq_sgd_update(dq_ctx* ctx, int b, int n, float* Z, long ldz,
                        const float* dZ, long lddz, float lr);

/* Sec. 4.3 / Table 4: the latent may be driven by other optimisers than plain SGD.  The paper prints neither rule;
 * both are the standard ones.  All matrices n x n fp32, updated in place (Z, m, v, buf); dZ: in.
 *
 * Adam with bias correction, step t >= 1 (DQ_ERR_SHAPE otherwise):
 *   m <- beta1 m + (1 - beta1) dZ,  v <- beta2 v + (1 - beta2) dZ^2,
 *   Z <- Z - lr * (m / (1 - beta1^t)) / (sqrt(v / (1 - beta2^t)) + eps).
 * SGD with momentum (heavy ball, no dampening):  buf <- mu buf + dZ,  Z <- Z - lr * buf. */
dq_status dq_adam_update(dq_ctx* ctx, int b, int n, float* Z, long ldz, const float* dZ, long lddz,
                         float* m, long ldm, float* v, long ldv, int step, float lr,
                         float beta1, float beta2, float eps);
dq_status dq_sgd_momentum_update(dq_ctx* ctx, int b, int n, float* Z, long ldz, const float* dZ, long lddz,
                                 float* buf, long ldbuf, float lr, float mu);

/* One QR-Orth step (the loop body of Alg. 1) with Adam in place of its SGD update; arguments as for
 * dq_calib_step and dq_adam_update (m, v: b stacked n x n matrices of optimiser state, zero before step 1). */
dq_status dq_calib_step_adam(dq_ctx* ctx, int b, int T, int n,
                             const void* X, dq_dtype x_dtype, long ldx,
                             float* Z, long ldz, float* m, long ldm, float* v, long ldv, int step,
                             float lr, float beta1, float beta2, float eps,
                             dq_reduce reduce, float* loss_dev, float* R_or_null, long ldr);

/* Alg. 3 (App. B.2), Cayley SGD with momentum: the optimiser the paper compares QR-Orth with (Sec. 5, optimiser
 * comparison).  It moves the rotation itself along the Cayley transform of a skew-symmetric W instead of
 * re-parametrising it through a latent.  Per problem, with R the algorithm's X_k, G = dL/dR and M its momentum buffer
 * (zero before the first update):
 *   M <- beta M - G;   W^ = M R^T - 1/2 R (R^T M R^T);   W = W^ - W^^T;   M <- W R;
 *   alpha = min(lr, 2 q / (||W||_F + eps));   Y = R + alpha M;   `iters` times  Y <- R + alpha/2 W (R + Y);   R <- Y.
 * (The paper's constants: q = 0.5, iters = 2, eps = 1e-8.)  R and M: in/out, b stacked n x n fp32; G: in.
 * alpha_dev_or_null: out, b DEVICE floats, the step size each problem took.  DQ_ERR_SHAPE for iters outside 0..64,
 * q <= 0 or eps < 0.  Workspace: dq_workspace_bytes(1, n, 1, ...). */
dq_status dq_cayley_update(dq_ctx* ctx, int b, int n, float* R, long ldr, const float* G, long ldg,
                           float* M, long ldm, float lr, float beta, float q, int iters, float eps,
                           float* alpha_dev_or_null);

/* One calibration step with that optimiser in place of QR-Orth: loss and G = dL/dR at the INPUT rotation (Alg. 1 lines
 * 8-9, as in dq_rotate_loss_grad), then dq_cayley_update of R.  No latent, no QR.  loss_dev: b DEVICE floats. */
dq_status dq_cayley_step(dq_ctx* ctx, int b, int T, int n, const void* X, dq_dtype x_dtype, long ldx,
                         float* R, long ldr, float* M, long ldm, float lr, float beta, float q, int iters,
                         float eps, dq_reduce reduce, float* loss_dev);

/* The matrix-core GEMMs the path is built from, exported for kernel-level parity tests:
 *   C (M x N, fp32) = alpha * op(A) op(B) + beta * C.
 * f32: A, B fp32; ta != 0 means A is stored K x M, tb != 0 means B is stored N x K.
 * bf16: A, B bf16, fp32 accumulate; ta/tb as above. */
dq_status dq_gemm_f32(dq_ctx* ctx, int M, int N, int K, float alpha,
                      const float* A, long lda, int ta, const float* B, long ldb, int tb,
                      float beta, float* C, long ldc);
dq_status dq_gemm_bf16(dq_ctx* ctx, int M, int N, int K,
                       const void* A, long lda, int ta, const void* B, long ldb, int tb,
                       float* C, long ldc);

/* ---- measurement -------------------------------------------------------------------- */

/* Kernel classes whose launches can be bracketed with HIP events on the context's stream. */
typedef enum {
    DQ_K_GEMM_F32 = 0,     /* fp32 matrix-core GEMM (QR trailing updates, forming R, backward) */
    DQ_K_GEMM_BF16 = 1,    /* bf16 matrix-core GEMM (X @ R, X^T @ dY)                          */
    DQ_K_WHIP = 2,         /* fused Whip loss + gradient pass                                  */
    DQ_K_PANEL = 3,        /* Householder panel factorisation                                  */
    DQ_K_SMALL = 4,        /* everything else (T factors, reductions, sign fix, conversions)   */
    DQ_K_COUNT = 5
} dq_kernel_class;

/* mask: bit k enables event bracketing of class k launches (0 switches profiling off).  Resets
 * the accumulated records. */
dq_status dq_profile_enable(dq_ctx* ctx, unsigned mask);

/* Waits for the stream and returns, for one class, the summed duration (ms) of the bracketed
 * launches since dq_profile_enable, their count, and the algorithmic flops and bytes the library
 * attributed to them.  Any out pointer may be null. */
dq_status dq_profile_read(dq_ctx* ctx, dq_kernel_class k, double* ms, long* launches,
                          double* flops, double* bytes);

#ifdef __cplusplus
}
#endif
#endif /* DARTQR_H */
