// Internal declarations shared by the translation units of libdartqr.so (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "dartqr.h"

namespace dq {

constexpr int kWave = 64;            // CDNA wavefront width
constexpr int kPanel = 64;           // QR panel width nb (columns aggregated into one compact-WY block)
constexpr int kTrsmBlock = 128;      // diagonal block size of the blocked triangular solve
constexpr int kTrsmOuter = 512;      // its outer block: columns solved before the rest of the matrix is updated once
constexpr int kMaxSplit = 64;        // upper bound on split-K partials
constexpr int kHeadDim = 128;         // matrix size served by the batched small-rotation path
constexpr int kHeadsChunk = 2048;     // tokens per workgroup of its fused rotate / loss / gradient kernel
constexpr int kLossPartials = 65536; // upper bound on workgroups of the Whip pass (one partial each)
constexpr int kAccumPanels = 4;      // panels whose reflectors are merged before they are applied to the accumulated R
constexpr int kCholMaxParts = 64;    // upper bound on the Gram partials of the tall-panel path

typedef uint16_t bf16_t;             // raw bfloat16 storage

inline __host__ __device__ long round_up(long x, long m) { return (x + m - 1) / m * m; }

// ---- profiling hook ---------------------------------------------------------------
struct Profiler;   // defined in dq_api.hip
struct LaunchScope {
    // Brackets the launches made during its lifetime with a pair of HIP events when the class is
    // enabled, and attributes `flops` / `bytes` of algorithmic work to it.
    LaunchScope(Profiler* p, hipStream_t s, int klass, double flops, double bytes);
    ~LaunchScope();
    Profiler* prof; hipStream_t stream; int klass; int slot;
};

// ---- fp32 matrix-core GEMM --------------------------------------------------------
struct GemmF32 {
    const float* A = nullptr; long lda = 0;
    const float* B = nullptr; long ldb = 0;
    float* C = nullptr; long ldc = 0;
    int M = 0, N = 0, K = 0;
    int ta = 0;            // A is stored K x M (the product uses its transpose)
    int tb = 0;            // B is stored N x K
    float alpha = 1.f, beta = 0.f;
    const float* alpha_dev = nullptr;   // non-null: alpha is multiplied by this device scalar
    // A's STORAGE is a block of Householder vectors: entry (r, c) is 0 for r < c, 1 for r == c and the
    // stored value for r > c (the stored upper part belongs to the triangular factor).
    int a_unit_lower = 0;
    // The first `b_unit_lower_cols` storage columns of B (tb == 0) get the same treatment.
    int b_unit_lower_cols = 0;
    // B(k, n) is known to vanish for k <= n (strictly lower triangular, tb == 0): K loop starts at the tile's n0.
    int b_strict_lower = 0;
    // split-K: z-th workgroup layer reduces k in [z*kchunk, (z+1)*kchunk) and writes C + z*split_stride
    int splits = 1; int kchunk = 0; long split_stride = 0;
    int cfg = -1;          // tile configuration (-1: chosen from the shape; 3: 64 x 64 tiles, K step 32)
    // batch > 1: that many independent products in one launch; problem i reads A + i*batch_a, B + i*batch_b and
    // writes C + i*batch_c (element offsets)
    int batch = 1; long batch_a = 0, batch_b = 0, batch_c = 0;
};
hipError_t launch_gemm_f32(const GemmF32& g, hipStream_t s);
int gemm_f32_tile_n(int M, int N);   // width of the workgroup tile the launcher picks

// ---- bf16 matrix-core GEMM (fp32 accumulate, fp32 out) ------------------------------
struct GemmBf16 {
    const bf16_t* A = nullptr; long lda = 0;
    const bf16_t* B = nullptr; long ldb = 0;
    float* C = nullptr; long ldc = 0;
    int M = 0, N = 0, K = 0;
    int ta = 0, tb = 0;    // as above
    int splits = 1; int kchunk = 0; long split_stride = 0;
    // a_kwrap > 0: the reduction index k runs over [0, 2*a_kwrap); A is read at k mod a_kwrap (columns
    // >= a_klim read as zero) while B supplies two planes [hi | lo] of a_kwrap columns each (tb == 1).
    // Used for X @ (R_hi + R_lo) with one pass over the accumulators.  Not combined with split-K.
    int a_kwrap = 0; int a_klim = 0;
    // whip_dyt != null: fused Whip epilogue (Eq. 4): dY^T (N x M bf16, leading dimension whip_ldt) and one partial sum
    // of exp(-|y|) per workgroup (gemm_bf16_whip_partials() doubles) are produced from the accumulators; C may then be
    // null.  Only for shapes gemm_bf16_deep_fits() accepts.
    bf16_t* whip_dyt = nullptr; long whip_ldt = 0; float whip_scale = 0.f; double* whip_partials = nullptr;
    // launch_gemm_bf16x3 only: element distance between the three planes of each operand, the epilogue
    // C = alpha * (A B^T) + beta * C, and b_strict_lower: B^T(k, n) vanishes for k <= n (K == N), the reduction of a tile
    // starts at its first column
    long a_plane = 0, b_plane = 0; float alpha = 1.f, beta = 0.f; int b_strict_lower = 0;
    const float* alpha_dev = nullptr;   // non-null: alpha is multiplied by this device scalar
};
hipError_t launch_gemm_bf16(const GemmBf16& g, hipStream_t s);
// fp32 product from three-plane bf16 splits of both operands (launch_split3_bf16), six plane pairs accumulated in fp32 on
// the bf16 matrix cores: C (M x N fp32) = alpha * A B^T + beta * C with A (M x K) and B (N x K) row-major planes.
// M and N multiples of 256, K of 64, 16-byte aligned rows and planes; anything else returns hipErrorInvalidValue.
// With b_strict_lower, splits = 2 halves every tile's reduction range: part z is written (alpha, beta as given) to
// C + z * split_stride and the caller sums the parts (launch_splitk_reduce).  A triangular product of 256 tiles or a few
// more is one workgroup per compute unit, and the longest tile sets the time, as long as the full product's; in halves, dealt out
// longest first, the compute units end up with about the same work each.
bool gemm_bf16x3_fits(int M, int N, int K);
hipError_t launch_gemm_bf16x3(const GemmBf16& g, hipStream_t s);
// out plane p (p = 0, 1, 2; at out + p * plane elements, leading dimension ldo) = p-th bf16 term of A (rows x cols
// fp32): a1 = bf16(a), a2 = bf16(a - a1), a3 = bf16(a - a1 - a2), round to nearest even; transpose != 0 writes the planes
// of A^T (cols x rows).
hipError_t launch_split3_bf16(const float* A, long lda, int rows, int cols, bf16_t* out, long ldo, long plane, int transpose,
                              hipStream_t s);
bool gemm_bf16_deep_fits(const GemmBf16& g);   // large round NT product: the unguarded deep-prefetch kernels apply
int gemm_bf16_whip_partials(const GemmBf16& g);   // workgroups (= partial sums) of the fused-epilogue launch for such a shape

// out (rows x cols, ldo) = alpha * sum_z part[z] + beta * out
hipError_t launch_splitk_reduce(const float* part, int splits, long stride, long ldp, int rows, int cols,
                                float alpha, float beta, float* out, long ldo, hipStream_t s);

// ---- ordering between streams by a device word ------------------------------------------
// The producing stream stores a growing value into the word after its work (a kernel of its own, or the first
// instructions of a kernel that follows that work in the same stream); the consuming stream polls the word (a kernel of
// its own in front of its work, or the first instructions of every workgroup of the consuming kernel).  Agent-scope
// release / acquire, so that what the producer wrote is read fresh.  Every poll is bounded by the device's constant-rate
// clock (100 MHz): past the limit it raises DQ_FLAG_SYNC_TIMEOUT and goes on, so every wavefront ends whatever the
// other stream does; once the bit is up, later polls return at once.
struct HandOver {
    const unsigned long long* wait_word = nullptr; unsigned long long wait_value = 0; long limit_us = 0;
    unsigned* flags = nullptr;
    unsigned long long* signal_word = nullptr; unsigned long long signal_value = 0;
};
__device__ __forceinline__ void handover_signal(unsigned long long* word, unsigned long long value) {
    __hip_atomic_store(word, value, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_AGENT);
}
// returns false if it gave up; one thread calls it
__device__ __forceinline__ bool handover_wait(const unsigned long long* word, unsigned long long value, long long limit_ticks,
                                              unsigned* flags) {
    if (flags != nullptr && (__hip_atomic_load(flags, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) & DQ_FLAG_SYNC_TIMEOUT))
        return false;
    const long long t0 = wall_clock64();
    for (;;) {
        if (__hip_atomic_load(word, __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_AGENT) >= value) return true;
        if (wall_clock64() - t0 > limit_ticks) break;
        __builtin_amdgcn_s_sleep(4);
    }
    if (flags != nullptr) atomicOr(flags, DQ_FLAG_SYNC_TIMEOUT);
    return false;
}
// *word = value once everything enqueued before on s has run
hipError_t launch_stream_signal(unsigned long long* word, unsigned long long value, hipStream_t s);
// what is enqueued after on s runs once *word >= value; gives up after limit_us (then DQ_FLAG_SYNC_TIMEOUT is or-ed
// into *flags and 1 stored to *timed_out, either may be null)
hipError_t launch_stream_wait(const unsigned long long* word, unsigned long long value, long limit_us, unsigned* flags,
                              unsigned long long* timed_out, hipStream_t s);

// ---- QR pieces --------------------------------------------------------------------
// Factor the m x jb panel at A (row-major, lda) in place: reflectors below the diagonal (unit diagonal
// implied), triangular factor on and above it; tau[0..jb).  vscratch: >= panel_scratch_floats(m) floats.
// tslices (kPanel*kPanel floats) receives the T factor of every column slice; *slice_width its width.
size_t panel_scratch_floats(int m);
hipError_t launch_qr_panel(float* A, long lda, int m, int jb, float* tau, float* vscratch, float* tslices,
                           int* slice_width, unsigned* flags, hipStream_t s);
// m x 64 panel (m >= 64) by CholeskyQR2 + Householder reconstruction on many compute units, in two calls.
// launch_cholqr_factor: everything up to the top 64 x 64 block: triangular factor and the first 64 rows of the
//   reflectors in A (as launch_qr_panel leaves them, except that row signs of the triangular factor may differ), T
//   (64 x 64, ld 64) in Tout, the first 64 rows of Yp = V T (m x 64, ld 64).  have_gram != 0: the first pass of the
//   panel (Cholesky factor of its Gram matrix, Q1 = A U1^-1 in q1 and the partials of Q1^T Q1) is already in the
//   scratch, left there by the previous panel's launch_cholqr_finish.
// launch_cholqr_finish: the rows of V and Yp below the block (none for m == 64).  lookahead != 0 (needs m >= 128):
//   it also applies the
//   panel's block reflector to the next 64 columns A[:, 64:128] (so these must have received every earlier update
//   before this call), and with next_gram != 0 leaves the first pass of the next panel A[64:, 64:128] behind
//   (Cholesky factor of its Gram matrix and the inverse, computed beside the update from quantities of before the
//   update; then Q1 in q1, which this call has read by then, and the partials of Q1^T Q1).  status: the device status
//   word (a bounded wait inside the kernel reports there).
// q1: m x 64 floats of scratch (also the panel kernel's reflector scratch); scratch: cholpanel_scratch_floats()
// floats; tau, tslices as for launch_qr_panel.  A panel that is too ill-conditioned for this route is factored by
// the Householder panel code inside the same launches (slow but rare; same outputs) and DQ_FLAG_ILLCOND_PANEL is
// or-ed into *status.
size_t cholpanel_scratch_floats();
bool cholpanel_supported(const float* A, long lda, int m, int jb);
hipError_t launch_cholqr_factor(float* A, long lda, int m, float* Tout, float* Yp, float* q1, float* scratch,
                                float* tau, float* tslices, unsigned* status, int have_gram, hipStream_t s);
// ho (may be null; only with lookahead != 0): the kernel that first reads the look-ahead columns polls ho->wait_word
// in every workgroup before it does (wait_word == null: no wait), and the kernel after it stores ho->signal_value to
// ho->signal_word when it starts, i.e. once the reflectors and Yp are complete (signal_word == null: no signal).
hipError_t launch_cholqr_finish(float* A, long lda, int m, float* Yp, float* q1, float* scratch, int lookahead,
                                int next_gram, unsigned* status, hipStream_t s, const HandOver* ho = nullptr);

// launch_cholqr_factor (have_gram != 0) and launch_cholqr_finish (lookahead != 0, next_gram != 0) as ONE launch whose
// workgroups hand over to each other through four 8-byte words at `words` (zero before the first use, then only
// growing): [0] and [2] take `epoch`, a value larger than any used before; [1] counts workgroups: `target` is the sum of
// cholqr_fused_workgroups(m) over every launch on these words so far, this one included; [3] counts the workgroups below
// the top block: `target_rows` is the sum of cholqr_fused_workgroups(m) - 1 likewise.  Polls give up after limit_us
// (DQ_FLAG_SYNC_TIMEOUT in *status).  cholqr_fused_workgroups(m) == 0: the panel does not fit this launch.
int cholqr_fused_workgroups(int m);
hipError_t launch_cholqr_fused(float* A, long lda, int m, float* Tout, float* Yp, float* q1, float* scratch, float* tau,
                               float* tslices, unsigned* status, unsigned long long* words, unsigned long long epoch,
                               unsigned long long target, unsigned long long target_rows, long limit_us, hipStream_t s,
                               const HandOver* ho);

// T (kPanel x kPanel, upper, zero beyond jb) of the compact-WY form from the slice T factors and the split-K
// partials of V^T [V | C] (gpart[z] at stride, leading dimension ldp: jb Gram columns, then nla columns of V^T C).
// Also W2out (jb x nla, ld kPanel) = T^T (V^T C).
hipError_t launch_tfactor(const float* gpart, int splits, long stride, long ldp, int jb, int nla,
                          const float* tslices, int slice_width, float* Tout, float* W2out, hipStream_t s);

// dst (rows x cols, ldd) = src (lds);  src == null writes zeros
hipError_t launch_copy2d(const float* src, long lds, float* dst, long ldd, int rows, int cols, hipStream_t s);
hipError_t launch_set_identity(float* A, long lda, int n, hipStream_t s);
hipError_t launch_fill_u32(unsigned* p, long count, unsigned v, hipStream_t s);
// s_j = sign(Afac[j][j]) (>= 0 -> +1);  R[:, j] *= s_j;  U = diag(s) * triu(Afac) (if U != null)
hipError_t launch_sign_normalise(const float* Afac, long lda, int n, float* R, long ldr, float* U, long ldu,
                                 unsigned* flags, hipStream_t s);

// ---- batched 128 x 128 rotations (all problems of a batch in one launch) -------------
// R (orthogonal, diag(U) >= 0) and U (optional) of b latents; problem i at Z + i*sz etc. (element strides).
hipError_t launch_heads_qr(int b, const float* Z, long ldz, long sz, float* R, long ldr, long sr, float* U, long ldu,
                           long su, unsigned* flags, hipStream_t s);
// loss[i] = scale * sum exp(-|X_i R_i|) and G_i = X_i^T dY_i for bf16 X_i (T x 128), fused.  Gpart needs
// b * heads_splits(T) * 128 * 128 floats, lpart b * heads_splits(T) doubles.
int heads_splits(int T);
hipError_t launch_heads_rlg(int b, int T, const bf16_t* X, long ldx, long sx, const float* R, long ldr, long sr,
                            float scale, float* Gpart, double* lpart, float* G, long ldg, long sg, float* loss,
                            unsigned* flags, hipStream_t s);

// Z = diag(sgn) H_n / sqrt(n), H_n the Sylvester Hadamard matrix (n a power of two)
hipError_t launch_hadamard_init(const float* sgn, int n, float* Z, long ldz, hipStream_t s);
// *count += number of entries of the T x n matrix Y with |y| > tau (count must hold the starting value)
hipError_t launch_outlier_count(const float* Y, long ldy, int T, int n, float tau, unsigned long long* count,
                                hipStream_t s);
// out row t = src row idx[t] (row_bytes a multiple of 16, 16-byte aligned rows); bad indices raise DQ_FLAG_BAD_INDEX
hipError_t launch_gather_rows(const void* src, long src_stride_bytes, int rows_in, const int* idx, int rows_out,
                              int row_bytes, void* out, long out_stride_bytes, unsigned* flags, hipStream_t s);

// ---- backward pieces --------------------------------------------------------------
// P = strict_lower(B - B^T); Mzero gets zeros everywhere (if non-null).
// batch > 1: that many problems in one launch, problem i at the given element strides.
hipError_t launch_skew_lower(const float* B, long ldb, int n, float* P, long ldp, float* Mzero, long ldm, hipStream_t s,
                             int batch = 1, long stride_b = 0, long stride_p = 0, long stride_m = 0);
// Inverse of every kTrsmBlock x kTrsmBlock diagonal block of the upper-triangular U: Uinv[blk] row-major, ld kTrsmBlock.
hipError_t launch_trinv_blocks(const float* U, long ldu, int n, float* Uinv, unsigned* flags, hipStream_t s,
                               int batch = 1, long stride_u = 0, long stride_inv = 0);
hipError_t launch_axpy2d(float* Z, long ldz, const float* D, long ldd, int n, float a, hipStream_t s);
// out (n / kTrsmOuter row-major blocks of kTrsmOuter x kTrsmOuter; n a multiple of kTrsmOuter) = the kTrsmBlock x kTrsmBlock
// inverses of launch_trinv_blocks on the block diagonal, zero elsewhere
hipError_t launch_place_diag_blocks(const float* inv, float* out, int n, hipStream_t s);
// Adam / heavy-ball updates of an n x n matrix in place (see include/dartqr.h); c1 = 1 / (1 - beta1^t),
// c2 = 1 / (1 - beta2^t) are formed on the host in double precision.
hipError_t launch_adam2d(float* Z, long ldz, const float* D, long ldd, float* m, long ldm, float* v, long ldv, int n,
                         float lr, float beta1, float beta2, float eps, float c1, float c2, hipStream_t s, int rows = -1);
hipError_t launch_momentum2d(float* Z, long ldz, const float* D, long ldd, float* buf, long ldb, int n, float lr,
                             float mu, hipStream_t s);

// ---- Cayley SGD pieces (Alg. 3, App. B.2) -------------------------------------------
// M <- beta M - G
hipError_t launch_cayley_momentum(float* M, long ldm, const float* G, long ldg, int n, float beta, hipStream_t s);
// W = What - What^T and partials[block] = sum of squares of this block's entries of W (cayley_skew_grid(n) blocks)
int cayley_skew_grid(int n);
hipError_t launch_cayley_skew(const float* What, long ldh, int n, float* W, long ldw, double* partials, hipStream_t s);
// alpha_dev[0] = min(lr, 2 q / (sqrt(sum of the partials) + eps)), alpha_dev[1] = alpha_dev[0] / 2
hipError_t launch_cayley_alpha(const double* partials, int count, float lr, float q, float eps, float* alpha_dev,
                               hipStream_t s);
// out = A + scale * B with scale = scale_host * (scale_dev ? *scale_dev : 1); out may alias A or B
hipError_t launch_add_scaled(float* out, long ldo, const float* A, long lda, const float* B, long ldb, int n,
                             float scale_host, const float* scale_dev, hipStream_t s);

// ---- rotate / Whip pieces ---------------------------------------------------------
// Split R into two bf16 planes and transpose:  RbT[j][k] = hi(R[k][j]),  RbT[j][koff + k] = lo(R[k][j]) with
// hi = bf16(r), lo = bf16(r - hi); columns k in [n, koff) of both planes are written as zero.  ldt >= 2*koff.
// dst (cols x rows, ldd) = src^T, src rows x cols (lds_); sizes multiples of 64, 16-byte aligned rows
hipError_t launch_transpose_bf16(const bf16_t* src, long lds_, int rows, int cols, bf16_t* dst, long ldd, hipStream_t s);
hipError_t launch_split_transpose_bf16(const float* R, long ldr, int n, bf16_t* RbT, long ldt, int koff, hipStream_t s);
// Fused Whip loss + gradient pass: partial sums to `partials` (double, one per workgroup), then
// launch_loss_finish adds them up: loss = scale * sum.  dy_is_bf16 selects the dtype of dY.
int whip_grid(long rows, int cols);
hipError_t launch_whip(const float* Y, long ldy, int T, int n, float scale, void* dY, int dy_is_bf16, long lddy,
                       double* partials, int grid, hipStream_t s, int batch = 1, long stride_y = 0, long stride_dy = 0);
hipError_t launch_loss_finish(const double* partials, int count, float scale, float* loss_dev, unsigned* flags,
                              hipStream_t s, int batch = 1);

// Row-wise objectives (1 variance, 2 kurtosis, 3 quantisation error): one partial per workgroup like the Whip pass.
int objective_grid(int T, int n);
hipError_t launch_objective(int objective, int bits, const float* Y, long ldy, int T, int n, float scale, void* dY,
                            int dy_is_bf16, long lddy, double* partials, int grid, hipStream_t s, int batch = 1,
                            long stride_y = 0, long stride_dy = 0);

}  // namespace dq
