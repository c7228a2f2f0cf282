// Tall panel factorisation spread over many compute units (a communication-avoiding replacement of the
// one-workgroup Householder panel for tall m x 64 panels of Alg. 2's blocked form):
//
//   1. CholeskyQR, twice:  G = A^T A = U1^T U1,  Q1 = A U1^-1,  G2 = Q1^T Q1 = U2^T U2,  Q = Q1 U2^-1,
//      Rf = U2 U1  (A = Q Rf, Q orthonormal to rounding when ||G2 - I|| is small; that is checked).
//   2. Householder reconstruction: with Q_top the first 64 rows of Q, an LU factorisation without pivoting of
//      Q_top - S (S = diag(s), s_j = -sign of the pivot met at step j, so every pivot has modulus >= 1) gives
//      Q - [S; 0] = V U_lu with V unit lower trapezoidal.  Then  I - V T V^T  with  T = -U_lu S V_top^-T  maps
//      [I; 0] S to Q, i.e. A = (I - V T V^T) [S Rf; 0]:  exactly the compact-WY form (V, T) and the triangular
//      factor S Rf that the Householder panel would hand to the rest of the blocked QR (up to row signs, which
//      the final sign normalisation removes).
//
// Everything that touches the m rows is a tall-skinny product on the matrix cores, spread over m / 128
// workgroups; the 64 x 64 work (sums of partials, Cholesky, LU, triangular inverses, small products) runs in
// one workgroup out of LDS.  Besides V, T and the triangular factor the route also returns Yp = V T (m x 64), the
// operand the trailing updates and the accumulation of the orthogonal factor multiply with.
// Between consecutive tall panels the first small step (Gram matrix, Cholesky, inverse) is taken off the chain of
// dependent kernels: it runs in one extra workgroup of the kernel that applies the previous panel's reflector to the
// panel's columns, from the Gram matrix of those columns BEFORE the update (see la_update_chol_kernel).
// When the check in step 1 fails (ill-conditioned or rank-deficient panel) the same one-workgroup kernel factors
// the untouched panel with the Householder panel code instead and builds T and Yp itself (slow, rare), so the
// launch sequence never depends on the data.
#include <stdlib.h>

#include "dq_internal.h"
#include "dq_small64.h"
#include "qr_panel_body.h"

namespace dq {
namespace {

constexpr int RT = 128;          // rows of one tile
constexpr int NSUM = 512;        // threads of the small-matrix kernels while they sum the partials

// rows [row0, row0 + 128) x 64 columns of X (leading dimension ldx, 16-byte aligned rows) -> Xs[r * LS + c];
// rows >= mrows read as zero.
__device__ __forceinline__ void load_tile(const float* __restrict__ X, long ldx, int row0, int mrows, float* Xs,
                                          int tid) {
    float4 v[8];
#pragma unroll
    for (int p = 0; p < 8; ++p) {
        const int r = p * 16 + (tid >> 4);
        const int gr = row0 + r;
        v[p] = (gr < mrows) ? *reinterpret_cast<const float4*>(X + (long)gr * ldx + 4 * (tid & 15))
                            : make_float4(0.f, 0.f, 0.f, 0.f);
    }
#pragma unroll
    for (int p = 0; p < 8; ++p) {
        float* d = Xs + (p * 16 + (tid >> 4)) * LS + 4 * (tid & 15);
        d[0] = v[p].x; d[1] = v[p].y; d[2] = v[p].z; d[3] = v[p].w;
    }
}

// 64 x 64 matrix (row-major, leading dimension 64) -> Ms[r * 64 + c]
__device__ __forceinline__ void load_small64(const float* __restrict__ Mg, float* Ms, int tid) {
#pragma unroll
    for (int p = 0; p < 4; ++p) {
        const int e = 4 * (tid + NTHR * p);
        *reinterpret_cast<float4*>(Ms + e) = *reinterpret_cast<const float4*>(Mg + e);
    }
}

// acc += (X^T X)[32 qi + ., 32 qj + .] over the 128 rows of the tile
__device__ __forceinline__ void gram_tile(const float* Xs, f32x16& acc, int qi, int qj, int lrow, int lk) {
#pragma unroll 8
    for (int r = 0; r < RT; r += 2) {
        const float a = Xs[(r + lk) * LS + 32 * qi + lrow];
        const float b = Xs[(r + lk) * LS + 32 * qj + lrow];
        acc = MFMA32(a, b, acc);
    }
}

__device__ __forceinline__ void store_partial(float* part, const f32x16& acc, int qi, int qj, int lrow, int lk) {
#pragma unroll
    for (int v = 0; v < 16; ++v) {
        const int i = 32 * qi + 8 * (v >> 2) + 4 * lk + (v & 3);
        part[i * B64 + 32 * qj + lrow] = acc[v];
    }
}

// rows [32 wave, 32 wave + 32) of the tile times the upper-triangular 64 x 64 matrix in Ms: two 32 x 32 results
__device__ __forceinline__ void mul_tile(const float* Xs, const float* Ms, f32x16& acc0, f32x16& acc1, int wave,
                                         int lrow, int lk) {
#pragma unroll 8
    for (int k0 = 0; k0 < 32; k0 += 2) {
        const float a = Xs[(32 * wave + lrow) * LS + k0 + lk];
        acc0 = MFMA32(a, Ms[(k0 + lk) * B64 + lrow], acc0);
        acc1 = MFMA32(a, Ms[(k0 + lk) * B64 + 32 + lrow], acc1);
    }
#pragma unroll 8
    for (int k0 = 32; k0 < 64; k0 += 2) {   // rows >= 32 of an upper-triangular factor only reach columns >= 32
        const float a = Xs[(32 * wave + lrow) * LS + k0 + lk];
        acc1 = MFMA32(a, Ms[(k0 + lk) * B64 + 32 + lrow], acc1);
    }
}

// part[blockIdx.x] (64 x 64) = sum over this workgroup's rows of A^T A
__global__ __launch_bounds__(NTHR) void ts_gram_kernel(const float* __restrict__ A, long lda, int m, int tiles_per_wg,
                                                       float* __restrict__ part) {
    __builtin_amdgcn_s_setprio(3);   // the panel chain is latency-critical: win issue slots from co-resident GEMM waves
    __shared__ float Xs[RT * LS];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int lrow = lane & 31, lk = lane >> 5;
    const int qi = wave >> 1, qj = wave & 1;
    f32x16 acc = zero16();
    for (int t = 0; t < tiles_per_wg; ++t) {
        const int row0 = (blockIdx.x * tiles_per_wg + t) * RT;
        if (row0 >= m) break;
        if (t > 0) __syncthreads();
        load_tile(A, lda, row0, m, Xs, tid);
        __syncthreads();
        gram_tile(Xs, acc, qi, qj, lrow, lk);
    }
    store_partial(part + (long)blockIdx.x * B64 * B64, acc, qi, qj, lrow, lk);
}

// Q1 = A Minv (written with leading dimension 64) and part[blockIdx.x] = Q1^T Q1 over this workgroup's rows
__global__ __launch_bounds__(NTHR) void ts_mul_gram_kernel(const float* __restrict__ A, long lda, int m,
                                                           int tiles_per_wg, const float* __restrict__ Minv,
                                                           float* __restrict__ Q1, float* __restrict__ part) {
    __builtin_amdgcn_s_setprio(3);   // the panel chain is latency-critical: win issue slots from co-resident GEMM waves
    __shared__ float Xs[RT * LS];
    __shared__ __attribute__((aligned(16))) float Ms[B64 * B64];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int lrow = lane & 31, lk = lane >> 5;
    const int qi = wave >> 1, qj = wave & 1;
    load_small64(Minv, Ms, tid);
    f32x16 acc = zero16();
    for (int t = 0; t < tiles_per_wg; ++t) {
        const int row0 = (blockIdx.x * tiles_per_wg + t) * RT;
        if (row0 >= m) break;
        if (t > 0) __syncthreads();
        load_tile(A, lda, row0, m, Xs, tid);
        __syncthreads();
        f32x16 q0 = zero16(), q1 = zero16();
        mul_tile(Xs, Ms, q0, q1, wave, lrow, lk);
        __syncthreads();
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int r = 32 * wave + 8 * (v >> 2) + 4 * lk + (v & 3);
            Xs[r * LS + lrow] = q0[v];
            Xs[r * LS + 32 + lrow] = q1[v];
            if (row0 + r < m) {
                Q1[(long)(row0 + r) * B64 + lrow] = q0[v];
                Q1[(long)(row0 + r) * B64 + 32 + lrow] = q1[v];
            }
        }
        __syncthreads();
        gram_tile(Xs, acc, qi, qj, lrow, lk);
    }
    store_partial(part + (long)blockIdx.x * B64 * B64, acc, qi, qj, lrow, lk);
}

// For the rows r >= row_off handled by this workgroup:  Vout[r][0:64] = Q1[r][:] Mm  and  Yout[r][0:64] = Q1[r][:] Mm2
// (both multipliers upper triangular, 64 x 64, ld 64; Yout has ld 64).  Skipped when *fb != 0.
__global__ __launch_bounds__(NTHR) void ts_mul_kernel(const float* __restrict__ Q1, int m, int row_off,
                                                      const float* __restrict__ Mm, const float* __restrict__ Mm2,
                                                      float* __restrict__ Vout, long ldv, float* __restrict__ Yout,
                                                      const unsigned* __restrict__ fb) {
    __builtin_amdgcn_s_setprio(3);   // the panel chain is latency-critical: win issue slots from co-resident GEMM waves
    if (*fb != 0u) return;
    __shared__ float Xs[RT * LS];
    __shared__ __attribute__((aligned(16))) float Ms[B64 * B64];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int lrow = lane & 31, lk = lane >> 5;
    const int row0 = row_off + blockIdx.x * RT;
    load_small64(Mm, Ms, tid);
    load_tile(Q1, B64, row0, m, Xs, tid);
    __syncthreads();
    {
        f32x16 q0 = zero16(), q1 = zero16();
        mul_tile(Xs, Ms, q0, q1, wave, lrow, lk);
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int r = row0 + 32 * wave + 8 * (v >> 2) + 4 * lk + (v & 3);
            if (r < m) {
                Vout[(long)r * ldv + lrow] = q0[v];
                Vout[(long)r * ldv + 32 + lrow] = q1[v];
            }
        }
    }
    __syncthreads();
    load_small64(Mm2, Ms, tid);
    __syncthreads();
    {
        f32x16 q0 = zero16(), q1 = zero16();
        mul_tile(Xs, Ms, q0, q1, wave, lrow, lk);
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int r = row0 + 32 * wave + 8 * (v >> 2) + 4 * lk + (v & 3);
            if (r < m) {
                Yout[(long)r * B64 + lrow] = q0[v];
                Yout[(long)r * B64 + 32 + lrow] = q1[v];
            }
        }
    }
}

// acc += (X^T C)[32 qi + ., 32 qj + .] over the 128 rows of two tiles
__device__ __forceinline__ void proj_tile(const float* Xs, const float* Cs, f32x16& acc, int qi, int qj, int lrow,
                                          int lk) {
#pragma unroll 8
    for (int r = 0; r < RT; r += 2) {
        const float a = Xs[(r + lk) * LS + 32 * qi + lrow];
        const float b = Cs[(r + lk) * LS + 32 * qj + lrow];
        acc = MFMA32(a, b, acc);
    }
}

// rows [32 wave, 32 wave + 32) of the tile times the full 64 x 64 matrix in Ws (row stride LS)
__device__ __forceinline__ void mul_tile_full(const float* Xs, const float* Ws, f32x16& acc0, f32x16& acc1, int wave,
                                              int lrow, int lk) {
#pragma unroll 8
    for (int k0 = 0; k0 < B64; k0 += 2) {
        const float a = Xs[(32 * wave + lrow) * LS + k0 + lk];
        acc0 = MFMA32(a, Ws[(k0 + lk) * LS + lrow], acc0);
        acc1 = MFMA32(a, Ws[(k0 + lk) * LS + 32 + lrow], acc1);
    }
}

// the first 64 rows of a reflector block as stored in the factored matrix -> unit lower triangular, in place in Xs
__device__ __forceinline__ void mask_unit_lower(float* Xs, int tid) {
#pragma unroll
    for (int q = 0; q < 16; ++q) {
        const int e = tid + NTHR * q, r = e >> 6, c = e & 63;
        if (c >= r) Xs[r * LS + c] = (c == r) ? 1.f : 0.f;
    }
}

// Last step of the tall-panel route fused with the first half of the look-ahead update of the next 64 columns
// C = A[:, 64:128]:  for its rows (workgroup 0: the top 64 rows; workgroup b >= 1: tpw tiles of 128 rows from row
// 64 + (b - 1) tpw 128) it writes V = Q1 Mm and Yp = Q1 Mm2 (rows >= 64; when *fb != 0 both were already written
// by the fallback and Yp is read back instead) and the partial  wpart[b] = Yp_rows^T C_rows  of the projection.
__global__ __launch_bounds__(NTHR) void ts_mul_proj_kernel(const float* __restrict__ Q1, int m,
                                                           const float* __restrict__ Mm, const float* __restrict__ Mm2,
                                                           float* A, long lda, float* Yp,
                                                           const unsigned* __restrict__ fb, int tpw,
                                                           float* __restrict__ wpart, float* __restrict__ gpart,
                                                           float* __restrict__ ctop, HandOver ho) {
    __builtin_amdgcn_s_setprio(3);   // the panel chain is latency-critical: win issue slots from co-resident GEMM waves
    __shared__ float Xs[RT * LS];
    __shared__ float Cs[RT * LS];
    if (ho.wait_word != nullptr) {   // the look-ahead columns must have received the previous trailing update
        if (threadIdx.x == 0) (void)handover_wait(ho.wait_word, ho.wait_value, (long long)ho.limit_us * 100, ho.flags);
        __syncthreads();
    }
    __shared__ __attribute__((aligned(16))) float Ms[B64 * B64];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int lrow = lane & 31, lk = lane >> 5;
    const int qi = wave >> 1, qj = wave & 1;
    const float* C = A + B64;
    f32x16 acc = zero16();
    f32x16 accg = zero16();          // gpart != null: C_rows^T C_rows of the look-ahead columns as they are BEFORE the update
    if (blockIdx.x == 0) {
        load_tile(Yp, B64, 0, B64, Xs, tid);
        load_tile(C, lda, 0, B64, Cs, tid);
        __syncthreads();
        proj_tile(Xs, Cs, acc, qi, qj, lrow, lk);
        if (gpart != nullptr) {
            gram_tile(Cs, accg, qi, qj, lrow, lk);
#pragma unroll
            for (int q = 0; q < 16; ++q) {
                const int e = tid + NTHR * q;
                ctop[e] = Cs[(e >> 6) * LS + (e & 63)];
            }
        }
    } else {
        const bool fell_back = *fb != 0u;
        for (int t = 0; t < tpw; ++t) {
            const int row0 = B64 + ((blockIdx.x - 1) * tpw + t) * RT;
            if (row0 >= m) break;
            if (t > 0) __syncthreads();
            if (!fell_back) {
                load_small64(Mm, Ms, tid);
                load_tile(Q1, B64, row0, m, Xs, tid);
                __syncthreads();
                {
                    f32x16 q0 = zero16(), q1 = zero16();
                    mul_tile(Xs, Ms, q0, q1, wave, lrow, lk);
#pragma unroll
                    for (int v = 0; v < 16; ++v) {
                        const int r = row0 + 32 * wave + 8 * (v >> 2) + 4 * lk + (v & 3);
                        if (r < m) {
                            A[(long)r * lda + lrow] = q0[v];
                            A[(long)r * lda + 32 + lrow] = q1[v];
                        }
                    }
                }
                __syncthreads();
                load_small64(Mm2, Ms, tid);
                __syncthreads();
                f32x16 q0 = zero16(), q1 = zero16();
                mul_tile(Xs, Ms, q0, q1, wave, lrow, lk);
                // each wavefront only read its own 32 rows of the tile: it may overwrite them with Yp right away
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int rl = 32 * wave + 8 * (v >> 2) + 4 * lk + (v & 3);
                    Xs[rl * LS + lrow] = q0[v];
                    Xs[rl * LS + 32 + lrow] = q1[v];
                    if (row0 + rl < m) {
                        Yp[(long)(row0 + rl) * B64 + lrow] = q0[v];
                        Yp[(long)(row0 + rl) * B64 + 32 + lrow] = q1[v];
                    }
                }
            } else {
                load_tile(Yp, B64, row0, m, Xs, tid);
            }
            load_tile(C, lda, row0, m, Cs, tid);
            __syncthreads();
            proj_tile(Xs, Cs, acc, qi, qj, lrow, lk);
            if (gpart != nullptr) gram_tile(Cs, accg, qi, qj, lrow, lk);
        }
    }
    store_partial(wpart + (long)blockIdx.x * B64 * B64, acc, qi, qj, lrow, lk);
    if (gpart != nullptr) store_partial(gpart + (long)blockIdx.x * B64 * B64, accg, qi, qj, lrow, lk);
}

// ------------------------------------------------------------------------------------------------------------
// 64 x 64 building blocks in LDS (row stride LS), one workgroup of 256 threads; every function ends with a
// barrier and must be called by all threads.

// Bm = sum of nparts (<= kCholMaxParts) partials of a symmetric 64 x 64 matrix (contiguous, 4096 floats each);
// called by NS threads, ZB partials in flight per thread and 16-byte piece (FULL: all four quadrants are read).  Only the quadrants on and above the diagonal are read (the lower-left 32 x 32 quadrant
// of Bm is set to zero): nothing downstream reads below the diagonal.  All loads of a thread are issued before
// the first add: a single workgroup is bound by latency here, not by bandwidth.
template <int NS = NSUM, int ZB = 16, bool FULL = false>
__device__ __forceinline__ void sum_partials(const float* __restrict__ part, int nparts, float* Bm, int tid) {
    constexpr int PER = B64 * B64 / 4 / NS;              // 16-byte pieces per thread
    float4 s[PER];
#pragma unroll
    for (int q = 0; q < PER; ++q) s[q] = make_float4(0.f, 0.f, 0.f, 0.f);
    for (int z0 = 0; z0 < nparts; z0 += ZB) {
        float4 t[PER][ZB];
#pragma unroll
        for (int q = 0; q < PER; ++q) {
            const int e = 4 * (tid + NS * q);
            const bool used = FULL || !((e >> 6) >= 32 && (e & 63) < 32);
#pragma unroll
            for (int z = 0; z < ZB; ++z)
                t[q][z] = (used && z0 + z < nparts)
                              ? *reinterpret_cast<const float4*>(part + (long)(z0 + z) * B64 * B64 + e)
                              : make_float4(0.f, 0.f, 0.f, 0.f);
        }
#pragma unroll
        for (int q = 0; q < PER; ++q)
#pragma unroll
            for (int z = 0; z < ZB; ++z) {
                s[q].x += t[q][z].x; s[q].y += t[q][z].y; s[q].z += t[q][z].z; s[q].w += t[q][z].w;
            }
    }
#pragma unroll
    for (int q = 0; q < PER; ++q) {
        const int e = 4 * (tid + NS * q);
        float* d = Bm + (e >> 6) * LS + (e & 63);
        d[0] = s[q].x; d[1] = s[q].y; d[2] = s[q].z; d[3] = s[q].w;
    }
    __syncthreads();
}

// The sum of n partials (contiguous, 4096 floats each) left in registers: thread tid of NS holds the 16-byte pieces
// 4 (tid + NS q).  FULL: all four quadrants; otherwise the lower-left 32 x 32 quadrant is skipped (zero).  No barrier.
template <int NS, int ZB, bool FULL = false>
__device__ __forceinline__ void sum_partials_regs(const float* __restrict__ part, int n, float4 (&s)[B64 * B64 / 4 / NS],
                                                  int tid) {
    constexpr int PER = B64 * B64 / 4 / NS;
#pragma unroll
    for (int q = 0; q < PER; ++q) s[q] = make_float4(0.f, 0.f, 0.f, 0.f);
    for (int z0 = 0; z0 < n; z0 += ZB) {
        float4 t[PER][ZB];
#pragma unroll
        for (int q = 0; q < PER; ++q) {
            const int e = 4 * (tid + NS * q);
            const bool used = FULL || !((e >> 6) >= 32 && (e & 63) < 32);
#pragma unroll
            for (int z = 0; z < ZB; ++z)
                t[q][z] = (used && z0 + z < n) ? *reinterpret_cast<const float4*>(part + (long)(z0 + z) * B64 * B64 + e)
                                               : make_float4(0.f, 0.f, 0.f, 0.f);
        }
#pragma unroll
        for (int q = 0; q < PER; ++q)
#pragma unroll
            for (int z = 0; z < ZB; ++z) {
                s[q].x += t[q][z].x; s[q].y += t[q][z].y; s[q].z += t[q][z].z; s[q].w += t[q][z].w;
            }
    }
}

// The two sums of la_update_chol_kernel's extra workgroup in the same batches of loads:  Wm = sum of the n partials at
// wp (all four quadrants),  Gm = sum of the n partials at gp (quadrants on and above the diagonal; the lower-left one is
// set to zero).  NS threads, ZB partials of each in flight per 16-byte piece; ends with a barrier.
template <int NS, int ZB>
__device__ __forceinline__ void sum_partials_pair(const float* __restrict__ wp, const float* __restrict__ gp, int n,
                                                  float* Wm, float* Gm, int tid) {
    constexpr int PER = B64 * B64 / 4 / NS;
    float4 sw[PER], sg[PER];
#pragma unroll
    for (int q = 0; q < PER; ++q) sw[q] = sg[q] = make_float4(0.f, 0.f, 0.f, 0.f);
    for (int z0 = 0; z0 < n; z0 += ZB) {
        float4 tw[PER][ZB], tg[PER][ZB];
#pragma unroll
        for (int q = 0; q < PER; ++q) {
            const int e = 4 * (tid + NS * q);
            const bool upper = !((e >> 6) >= 32 && (e & 63) < 32);
#pragma unroll
            for (int z = 0; z < ZB; ++z) {
                const bool in = z0 + z < n;
                tw[q][z] = in ? *reinterpret_cast<const float4*>(wp + (long)(z0 + z) * B64 * B64 + e)
                              : make_float4(0.f, 0.f, 0.f, 0.f);
                tg[q][z] = (in && upper) ? *reinterpret_cast<const float4*>(gp + (long)(z0 + z) * B64 * B64 + e)
                                         : make_float4(0.f, 0.f, 0.f, 0.f);
            }
        }
#pragma unroll
        for (int q = 0; q < PER; ++q)
#pragma unroll
            for (int z = 0; z < ZB; ++z) {
                sw[q].x += tw[q][z].x; sw[q].y += tw[q][z].y; sw[q].z += tw[q][z].z; sw[q].w += tw[q][z].w;
                sg[q].x += tg[q][z].x; sg[q].y += tg[q][z].y; sg[q].z += tg[q][z].z; sg[q].w += tg[q][z].w;
            }
    }
#pragma unroll
    for (int q = 0; q < PER; ++q) {
        const int e = 4 * (tid + NS * q);
        float* dw = Wm + (e >> 6) * LS + (e & 63);
        float* dg = Gm + (e >> 6) * LS + (e & 63);
        dw[0] = sw[q].x; dw[1] = sw[q].y; dw[2] = sw[q].z; dw[3] = sw[q].w;
        dg[0] = sg[q].x; dg[1] = sg[q].y; dg[2] = sg[q].z; dg[3] = sg[q].w;
    }
    __syncthreads();
}

// Rank-8 update on the matrix cores of the 64 x 64 matrix Wm held in LDS (row stride LS), for the entries with
// row >= lim and column >= lim only:  Wm[i][j] -= sum_{r<8} Lc(i, k0 + r) * Wm[k0 + r][j],  where Lc(i, k) is
// Wm[i][k] (SYM = false: the multipliers sit in columns k0.. of the same matrix) or Wm[k][i] (SYM = true: the
// symmetric case, multipliers are the transposed block row).  One 32 x 32 quadrant per wavefront.
template <bool SYM>
__device__ __forceinline__ void rank8_update(float* Wm, int k0, int lim, int qi, int qj, int lrow, int lk) {
    if (32 * (qi + 1) <= lim || 32 * (qj + 1) <= lim) return;          // quadrant entirely finished
    if (SYM && qi > qj) return;                                        // below the diagonal: never read
    const int i = 32 * qi + lrow, j = 32 * qj + lrow;
    float a[4], b[4];
    f32x16 acc;
    // all 24 values are requested before the first one is used (one wavefront per SIMD: nothing else hides the latency)
#pragma unroll
    for (int s4 = 0; s4 < 4; ++s4) {
        const int k = k0 + 2 * s4 + lk;
        a[s4] = SYM ? Wm[k * LS + i] : Wm[i * LS + k];
        b[s4] = Wm[k * LS + j];
    }
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[v] = Wm[(32 * qi + 8 * (v >> 2) + 4 * lk + (v & 3)) * LS + j];
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int s4 = 0; s4 < 4; ++s4) {
        a[s4] = (i >= lim) ? -a[s4] : 0.f;
        b[s4] = (j >= lim) ? b[s4] : 0.f;
    }
#pragma unroll
    for (int s4 = 0; s4 < 4; ++s4) acc = MFMA32(a[s4], b[s4], acc);
#pragma unroll
    for (int v = 0; v < 16; ++v) Wm[(32 * qi + 8 * (v >> 2) + 4 * lk + (v & 3)) * LS + j] = acc[v];
}

__device__ __forceinline__ float lane_value(float v, int l) {
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), l));
}

// In place: the upper triangle of the symmetric positive definite G becomes U with G = U^T U; the strict lower
// triangle is zeroed.  Blocked by 8.  The first wavefront holds the block row k0 .. k0+7 in registers, one column per
// lane, and factors it with lane broadcasts only (the diagonal block and the block row to its right in the same
// eight steps); then a rank-8 update of the rest on the matrix cores by all four wavefronts.
__device__ __forceinline__ void chol_upper_64(float* G, int tid) {
    const int lane = tid & 63;
    // (kept as a loop: the routine runs once per launch, from a cold instruction cache, and eight copies of its body
    // cost more to fetch than the loop control costs to execute)
#pragma unroll 1
    for (int k0 = 0; k0 < B64; k0 += 8) {
        if (tid < 64) {
            float p[8];
#pragma unroll
            for (int r = 0; r < 8; ++r) p[r] = G[(k0 + r) * LS + lane];
#pragma unroll
            for (int r = 0; r < 8; ++r) {
                // hardware reciprocal square root (1 ulp): U only has to be consistent with the inverse formed from it
                const float id = __builtin_amdgcn_rsqf(lane_value(p[r], k0 + r));
                p[r] *= id;
#pragma unroll
                for (int i = r + 1; i < 8; ++i) p[i] -= lane_value(p[r], k0 + i) * p[r];
            }
#pragma unroll
            for (int r = 0; r < 8; ++r)
                if (lane >= k0 + r) G[(k0 + r) * LS + lane] = p[r];
        }
        __syncthreads();
        rank8_update<true>(G, k0, k0 + 8, (tid >> 7) & 1, (tid >> 6) & 1, tid & 31, (tid >> 5) & 1);
        __syncthreads();
    }
#pragma unroll
    for (int q = 0; q < 16; ++q) {
        const int e = tid + NTHR * q;
        if ((e & 63) < (e >> 6)) G[(e >> 6) * LS + (e & 63)] = 0.f;
    }
    __syncthreads();
}

// In place LU without pivoting of W - diag(s), where s_j = -1 if the pivot met at step j is >= 0 and +1 otherwise
// (decided on the partially eliminated matrix), so that each pivot has modulus >= 1.  On return the strict lower
// triangle holds L (unit diagonal implied), the upper triangle U, and sg[0..64) the signs.
// Blocked by 8.  The first wavefront holds the block column k0 .. k0+7 in registers, one row per lane, and eliminates
// it with lane broadcasts.  At the same time the second wavefront holds the block row k0 .. k0+7, one column per lane,
// and runs the same eight elimination steps on it: on the 8 x 8 diagonal block both wavefronts apply the same
// operations to the same values (fused multiply-adds written out, so that the two cannot be contracted differently),
// hence meet the same pivots, signs and multipliers; the first one stores the diagonal block and L, the second one
// the block row of U to the right of it.  Then a rank-8 update on the matrix cores.
// The rows of the 8 x 8 diagonal block are stored one step late: while the first wavefront eliminates the block column,
// the second one still reads the diagonal block as it was (nothing orders the two before the barrier), and the rank-8
// update that follows rewrites every entry of its quadrants, this block included.  At the top of the next step nobody
// reads or writes the block.  In the last step the second wavefront has nothing to do and the block is stored at once.
__device__ __forceinline__ void lu_signed_64(float* W, float* sg, int tid) {
    const int lane = tid & 63, wave = tid >> 6;
    float pd[8];                                   // first wavefront, lanes k0 .. k0 + 7: their rows of the diagonal block
#pragma unroll
    for (int c = 0; c < 8; ++c) pd[c] = 0.f;
#pragma unroll 1
    for (int k0 = 0; k0 < B64; k0 += 8) {
        if (wave == 0) {
            if (k0 > 0 && lane >= k0 - 8 && lane < k0) {
#pragma unroll
                for (int c = 0; c < 8; ++c) W[lane * LS + k0 - 8 + c] = pd[c];
            }
            float p[8];
#pragma unroll
            for (int c = 0; c < 8; ++c) p[c] = W[lane * LS + k0 + c];
#pragma unroll
            for (int c = 0; c < 8; ++c) {
                const int pr = k0 + c;
                const float piv = lane_value(p[c], pr);
                const float sv = piv >= 0.f ? -1.f : 1.f;
                const float pv = piv - sv;
                const float inv = __builtin_amdgcn_rcpf(pv);
                const bool below = lane > pr;
                if (lane == pr) { p[c] = pv; sg[pr] = sv; }
                p[c] = below ? p[c] * inv : p[c];
#pragma unroll
                for (int c2 = c + 1; c2 < 8; ++c2) {
                    const float u = lane_value(p[c2], pr);
                    p[c2] = below ? __builtin_fmaf(-p[c], u, p[c2]) : p[c2];
                }
            }
            if (lane >= k0 + 8 || (lane >= k0 && k0 + 8 == B64)) {
#pragma unroll
                for (int c = 0; c < 8; ++c) W[lane * LS + k0 + c] = p[c];
            }
#pragma unroll
            for (int c = 0; c < 8; ++c) pd[c] = p[c];
        } else if (wave == 1 && k0 + 8 < B64) {
            float q[8];
#pragma unroll
            for (int r = 0; r < 8; ++r) q[r] = W[(k0 + r) * LS + lane];
#pragma unroll
            for (int r = 0; r < 7; ++r) {
                const int pr = k0 + r;
                const float piv = lane_value(q[r], pr);
                const float sv = piv >= 0.f ? -1.f : 1.f;
                const float inv = __builtin_amdgcn_rcpf(piv - sv);
#pragma unroll
                for (int i = r + 1; i < 8; ++i) {
                    const float l = lane_value(q[i], pr) * inv;
                    q[i] = __builtin_fmaf(-l, q[r], q[i]);     // (lanes k0 .. pr hold no longer needed entries)
                }
            }
            if (lane >= k0 + 8) {
#pragma unroll
                for (int r = 1; r < 8; ++r) W[(k0 + r) * LS + lane] = q[r];
            }
        }
        __syncthreads();
        rank8_update<false>(W, k0, k0 + 8, (tid >> 7) & 1, (tid >> 6) & 1, tid & 31, (tid >> 5) & 1);
        __syncthreads();
    }
}

// Second half of the look-ahead update:  W2 = sum of the nproj partials,  C -= V W2  for C = A[:, 64:128] (same row
// split as ts_mul_proj_kernel: workgroups 0 .. nproj - 1).
// gpart != null: one more workgroup (index nproj) runs BESIDE them and does the first small step of the NEXT panel
// (rows >= 64 of the updated C), so that this step is off the chain of dependent kernels.  It needs the Gram matrix of
// rows that the other workgroups are still updating; the block reflector H = I - V T V^T is orthogonal, so over all m
// rows  C'^T C' = C^T C  for C' = H^T C, and the rows >= 64 of C' have
//     G = C^T C - C'_top^T C'_top,   C'_top = C_top - V_top W2  (the first 64 rows),
// with C^T C summed from the partials that ts_mul_proj_kernel formed from the columns BEFORE the update (gpart, nproj
// of them) and C_top as it saved it (ctop).  Then U1 = chol(G) and its inverse, as chol_inv_kernel.  The difference
// between G and the Gram matrix of the stored rows is of the order of the rounding of H (1e-7 relative), like the
// rounding of a directly summed Gram matrix; what CholeskyQR needs from G is checked after its first pass as before.
template <int NT>
__global__ __launch_bounds__(NT) void la_update_chol_kernel(float* A, long lda, int m,
                                                              const float* __restrict__ wpart, int nproj, int tpw,
                                                              float* gpart,
                                                              const float* __restrict__ ctop, float* __restrict__ U1,
                                                              float* U1inv, float* __restrict__ Q1next,
                                                              unsigned long long* ready, unsigned* status, HandOver ho) {
    __builtin_amdgcn_s_setprio(3);   // the panel chain is latency-critical: win issue slots from co-resident GEMM waves
    // the kernel before this one completed the panel's reflectors and Yp: the other streams may go on
    if (ho.signal_word != nullptr && blockIdx.x == 0 && threadIdx.x == 0) handover_signal(ho.signal_word, ho.signal_value);
    __shared__ float Xs[RT * LS];
    __shared__ __attribute__((aligned(16))) float Ws[B64 * LS];
    __shared__ float Gs[B64 * LS];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int lrow = lane & 31, lk = lane >> 5;
    const int qi = (wave >> 1) & 1, qj = wave & 1;
    // launched with NT >= NTHR threads for the sake of the extra workgroup's sums; the updating workgroups use NTHR of them
    const bool extra = gpart != nullptr && (int)blockIdx.x == nproj;
    if (!extra && tid >= NTHR) return;
    if (!extra) {   // W2: 4 sixteen-byte pieces per thread, partials in groups of 8 (all loads of a group in flight)
        float4 s4[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) s4[q] = make_float4(0.f, 0.f, 0.f, 0.f);
        for (int z0 = 0; z0 < nproj; z0 += 8) {
            float4 t[4][8];
#pragma unroll
            for (int q = 0; q < 4; ++q)
#pragma unroll
                for (int z = 0; z < 8; ++z)
                    t[q][z] = (z0 + z < nproj)
                                  ? *reinterpret_cast<const float4*>(wpart + (long)(z0 + z) * B64 * B64 + 4 * (tid + NTHR * q))
                                  : make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
            for (int q = 0; q < 4; ++q)
#pragma unroll
                for (int z = 0; z < 8; ++z) {
                    s4[q].x += t[q][z].x; s4[q].y += t[q][z].y; s4[q].z += t[q][z].z; s4[q].w += t[q][z].w;
                }
        }
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int e = 4 * (tid + NTHR * q);
            float* d = Ws + (e >> 6) * LS + (e & 63);
            d[0] = s4[q].x; d[1] = s4[q].y; d[2] = s4[q].z; d[3] = s4[q].w;
        }
    }
    float* C = A + B64;
    if (extra) {
        // ---- the next panel's U1 = chol(G), U1^-1
        float* S0 = Xs;               // V_top
        float* S1 = Xs + B64 * LS;    // C_top, then C'_top
        // both sums with all NT threads: W2 (summed in another order than the updating workgroups sum it, which moves G
        // by rounding only) and C^T C over all rows (upper quadrants)
        // the two 64 x 64 blocks needed after the sums are requested first: they arrive meanwhile
        float4 vt[4], ct[4];
        if (tid < NTHR) {
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int e = 4 * (tid + NTHR * q);
                vt[q] = *reinterpret_cast<const float4*>(A + (long)(e >> 6) * lda + (e & 63));
                ct[q] = *reinterpret_cast<const float4*>(ctop + e);
            }
        }
        sum_partials_pair<NT, NT == NTHR ? 4 : 11>(wpart, gpart, nproj, Ws, Gs, tid);
        if (tid >= NTHR) return;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int e = 4 * (tid + NTHR * q);
            float* d0 = S0 + (e >> 6) * LS + (e & 63);
            float* d1 = S1 + (e >> 6) * LS + (e & 63);
            d0[0] = vt[q].x; d0[1] = vt[q].y; d0[2] = vt[q].z; d0[3] = vt[q].w;
            d1[0] = ct[q].x; d1[1] = ct[q].y; d1[2] = ct[q].z; d1[3] = ct[q].w;
        }
        __syncthreads();
        const f32x16 vw = lds_mma<2>(S0, Ws, nullptr, qi, qj, 0, B64, lrow, lk);   // V_top (unit lower) W2
        __syncthreads();
#pragma unroll
        for (int v = 0; v < 16; ++v) S1[(32 * qi + 8 * (v >> 2) + 4 * lk + (v & 3)) * LS + 32 * qj + lrow] -= vw[v];
        __syncthreads();
        if (qi <= qj) {
            f32x16 gt = zero16();                 // (C'_top^T C'_top)[32 qi + ., 32 qj + .]
#pragma unroll 8
            for (int r = 0; r < B64; r += 2)
                gt = MFMA32(S1[(r + lk) * LS + 32 * qi + lrow], S1[(r + lk) * LS + 32 * qj + lrow], gt);
#pragma unroll
            for (int v = 0; v < 16; ++v) Gs[(32 * qi + 8 * (v >> 2) + 4 * lk + (v & 3)) * LS + 32 * qj + lrow] -= gt[v];
        }
        __syncthreads();
        chol_upper_64(Gs, tid);
        tri_inv_upper_64<false>(Gs, Ws, tid);
#pragma unroll
        for (int q = 0; q < 16; ++q) {
            const int e = tid + NTHR * q;
            U1[e] = Gs[(e >> 6) * LS + (e & 63)];
            U1inv[e] = Ws[(e >> 6) * LS + (e & 63)];
        }
        __syncthreads();                       // every thread's part of U1^-1 is written: the other workgroups may use it
        if (tid == 0) handover_signal(ready, 1ull);
        return;
    }
    if (blockIdx.x == 0) {
        load_tile(A, lda, 0, B64, Xs, tid);
        __syncthreads();
        mask_unit_lower(Xs, tid);
        __syncthreads();
        f32x16 q0 = zero16(), q1 = zero16();
        mul_tile_full(Xs, Ws, q0, q1, wave, lrow, lk);
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int r = 32 * wave + 8 * (v >> 2) + 4 * lk + (v & 3);
            if (r < B64) {
                C[(long)r * lda + lrow] -= q0[v];
                C[(long)r * lda + 32 + lrow] -= q1[v];
            }
        }
        return;
    }
    for (int t = 0; t < tpw; ++t) {
        const int row0 = B64 + ((blockIdx.x - 1) * tpw + t) * RT;
        if (row0 >= m) break;
        if (t > 0) __syncthreads();
        load_tile(A, lda, row0, m, Xs, tid);
        __syncthreads();
        f32x16 q0 = zero16(), q1 = zero16();
        mul_tile_full(Xs, Ws, q0, q1, wave, lrow, lk);
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int r = row0 + 32 * wave + 8 * (v >> 2) + 4 * lk + (v & 3);
            if (r < m) {
                C[(long)r * lda + lrow] -= q0[v];
                C[(long)r * lda + 32 + lrow] -= q1[v];
            }
        }
    }
    if (gpart == nullptr) return;
    // ---- the next panel's second step for the rows this workgroup has just updated (what ts_mul_gram_kernel does):
    // Q1 = A_next U1^-1 and the partials of Q1^T Q1, once the extra workgroup has U1^-1.  The workgroups of a launch
    // run at the same time (34 or 66 of them on 256 compute units), the extra one waits for nobody, and the poll is
    // bounded like the polls between streams.
    __syncthreads();                           // the stores of the updated rows precede their reads below; Ws is free
    if (tid == 0) (void)handover_wait(ready, 1ull, 100LL * 1000 * 1000, status);
    __syncthreads();
    float* Ms = Ws;                            // 64 x 64, leading dimension 64
    load_small64(U1inv, Ms, tid);
    const float* An = A + (long)B64 * lda + B64;
    const int mn = m - B64;
    f32x16 acc = zero16();
    for (int t = 0; t < tpw; ++t) {
        const int row0 = ((blockIdx.x - 1) * tpw + t) * RT;
        if (row0 >= mn) break;
        __syncthreads();
        load_tile(An, lda, row0, mn, Xs, tid);
        __syncthreads();
        f32x16 q0 = zero16(), q1 = zero16();
        mul_tile(Xs, Ms, q0, q1, wave, lrow, lk);
        __syncthreads();
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int r = 32 * wave + 8 * (v >> 2) + 4 * lk + (v & 3);
            Xs[r * LS + lrow] = q0[v];
            Xs[r * LS + 32 + lrow] = q1[v];
            if (row0 + r < mn) {
                Q1next[(long)(row0 + r) * B64 + lrow] = q0[v];
                Q1next[(long)(row0 + r) * B64 + 32 + lrow] = q1[v];
            }
        }
        __syncthreads();
        gram_tile(Xs, acc, qi, qj, lrow, lk);
    }
    store_partial(gpart + (long)(blockIdx.x - 1) * B64 * B64, acc, qi, qj, lrow, lk);
}

// First small step: U1 = chol(sum of partials of A^T A) and its inverse, both 64 x 64 (leading dimension 64).
__global__ __launch_bounds__(NSUM) void chol_inv_kernel(const float* __restrict__ part, int nparts,
                                                        float* __restrict__ U1, float* __restrict__ U1inv) {
    __builtin_amdgcn_s_setprio(3);   // the panel chain is latency-critical: win issue slots from co-resident GEMM waves
    __shared__ float B0[B64 * LS];
    __shared__ float B1[B64 * LS];
    const int tid = threadIdx.x;
    sum_partials(part, nparts, B0, tid);
    if (tid >= NTHR) return;                    // the extra wavefronts only help to fetch the partials
    chol_upper_64(B0, tid);
    tri_inv_upper_64<false>(B0, B1, tid);
#pragma unroll
    for (int q = 0; q < 16; ++q) {
        const int e = tid + NTHR * q;
        U1[e] = B0[(e >> 6) * LS + (e & 63)];
        U1inv[e] = B1[(e >> 6) * LS + (e & 63)];
    }
}

// Builds what the Householder panel code does not return itself: T of the block reflector from the reflectors in
// the panel (m x 64 at A, unit lower trapezoidal) and tau, by the column recurrence
//   T[0:j, j] = -tau_j T[0:j, 0:j] (V[:, 0:j]^T v_j),  T[j, j] = tau_j,
// and Yp = V T.  One workgroup of NTHR threads; Bs: 3 * 64 * LS floats of LDS.  Slow path.
__device__ void fallback_finish(const float* __restrict__ A, long lda, int m, const float* __restrict__ tau,
                                float* __restrict__ Tout, float* __restrict__ Yp, float* Bs, int tid) {
    const int lane = tid & 63, wave = tid >> 6, lrow = lane & 31, lk = lane >> 5;
    const int qi = wave >> 1, qj = wave & 1;
    float* Xs = Bs;                        // a 128-row tile (2 * 64 * LS floats)
    float* Ms = Bs + 2 * B64 * LS;         // T, row stride 64
    f32x16 acc = zero16();
    for (int row0 = 0; row0 < m; row0 += RT) {
        if (row0 > 0) __syncthreads();
        load_tile(A, lda, row0, m, Xs, tid);
        __syncthreads();
        if (row0 == 0) {
#pragma unroll
            for (int q = 0; q < 16; ++q) {
                const int e = tid + NTHR * q, r = e >> 6, c = e & 63;
                if (c >= r) Xs[r * LS + c] = (c == r) ? 1.f : 0.f;
            }
            __syncthreads();
        }
        gram_tile(Xs, acc, qi, qj, lrow, lk);
    }
    __syncthreads();
    acc_to_lds(acc, Xs, qi, qj, lrow, lk);                 // G = V^T V
#pragma unroll
    for (int q = 0; q < 16; ++q) Ms[tid + NTHR * q] = 0.f;
    __syncthreads();
    for (int j = 0; j < B64; ++j) {
        const float tj = tau[j];
        if (tid < j) {
            float z = 0.f;
            for (int k = tid; k < j; ++k) z += Ms[tid * B64 + k] * Xs[k * LS + j];
            Ms[tid * B64 + j] = -tj * z;                   // column j is not read during this step
        } else if (tid == j) {
            Ms[j * B64 + j] = tj;
        }
        __syncthreads();
    }
#pragma unroll
    for (int q = 0; q < 16; ++q) Tout[tid + NTHR * q] = Ms[tid + NTHR * q];
    for (int row0 = 0; row0 < m; row0 += RT) {
        __syncthreads();
        load_tile(A, lda, row0, m, Xs, tid);
        __syncthreads();
        if (row0 == 0) {
#pragma unroll
            for (int q = 0; q < 16; ++q) {
                const int e = tid + NTHR * q, r = e >> 6, c = e & 63;
                if (c >= r) Xs[r * LS + c] = (c == r) ? 1.f : 0.f;
            }
            __syncthreads();
        }
        f32x16 q0 = zero16(), q1 = zero16();
        mul_tile(Xs, Ms, q0, q1, wave, lrow, lk);
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int r = row0 + 32 * wave + 8 * (v >> 2) + 4 * lk + (v & 3);
            if (r < m) {
                Yp[(long)r * B64 + lrow] = q0[v];
                Yp[(long)r * B64 + 32 + lrow] = q1[v];
            }
        }
    }
}

// Second small step (see the head of this file).  Inputs: partials of G2 = Q1^T Q1, the first 64 rows of Q1, U1.
// When the orthogonality check passes (*fb = 0) it writes the top 64 x 64 block of the panel (V_top strictly below
// the diagonal, S U2 U1 on and above it), T (64 x 64, ld 64), the first 64 rows of Yp = V T, and the two multipliers
// for the rows below the block: Mm = (U_lu U2)^-1 (V = Q1 Mm) and Mm2 = Mm T (Yp = Q1 Mm2).
// Otherwise (*fb = 1, DQ_FLAG_ILLCOND_PANEL raised) the workgroup factors the whole panel with the Householder
// panel code and writes V, the triangular factor, tau, T and all of Yp itself.
// The body: NSUM threads enter, those beyond the first NTHR return once the partials are summed (they take part in no
// later barrier); Bs: 5 * 64 * LS floats of LDS, sg: 64, redw: 4.
__device__ __forceinline__ void hr_finish_body(const float* __restrict__ part, int nparts, float* q1,
                                               const float* __restrict__ U1, float* A, long lda, int m,
                                               float* __restrict__ Tout, float* __restrict__ Yp,
                                               float* __restrict__ Mm, float* __restrict__ Mm2,
                                               float* __restrict__ tau, float* __restrict__ tslices,
                                               unsigned* __restrict__ fb, unsigned* __restrict__ status, float* Bs,
                                               float* sg, float* redw) {
    float* B0 = Bs;
    float* B1 = Bs + B64 * LS;
    float* B2 = Bs + 2 * B64 * LS;
    float* B3 = Bs + 3 * B64 * LS;
    float* B4 = Bs + 4 * B64 * LS;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int lrow = lane & 31, lk = lane >> 5;
    const int qi = (wave >> 1) & 1, qj = wave & 1;

    // U1 and the top block of Q1 are needed well after the partials are summed: requested now, they arrive meanwhile
    float u1r[16], q1r[16];
    if (tid < NTHR) {
#pragma unroll
        for (int q = 0; q < 16; ++q) { u1r[q] = U1[tid + NTHR * q]; q1r[q] = q1[tid + NTHR * q]; }
    }
    sum_partials(part, nparts, B0, tid);
    {   // ||G2 - I||_F^2 must be small: then Q1 is well conditioned and the second pass gives orthonormal columns
        if (tid < NTHR) {
            float dev = 0.f;
#pragma unroll
            for (int q = 0; q < 16; ++q) {
                const int e = tid + NTHR * q;
                const int i = e >> 6, j = e & 63;
                const float x = B0[i * LS + j] - ((i == j) ? 1.f : 0.f);
                if (j >= i) dev += (j > i ? 2.f : 1.f) * x * x;     // only the upper triangle was summed
            }
#pragma unroll
            for (int off = 32; off > 0; off >>= 1) dev += __shfl_xor(dev, off);
            if (lane == 0) redw[wave] = dev;
        }
        __syncthreads();
        const float total = redw[0] + redw[1] + redw[2] + redw[3];
        const bool ok = total < 0.25f;          // false for NaN as well
        if (tid == 0) *fb = ok ? 0u : 1u;
        if (!ok) {
            if (tid == 0) atomicOr(status, DQ_FLAG_ILLCOND_PANEL);
            // q1 doubles as the packed reflector scratch of the panel code (Q1 is dead now)
            qr_panel_body<NSUM, 16, 4, 16>(A, lda, m, B64, tau, q1, tslices, status, 1);
            __syncthreads();
            unpack_reflectors_body(A, lda, m, B64, q1, NSUM * 16, 4, 1, (long)tid, (long)NSUM);
            __syncthreads();
            if (tid >= NTHR) return;
            fallback_finish(A, lda, m, tau, Tout, Yp, Bs, tid);
            return;
        }
    }
    if (tid >= NTHR) return;                    // the extra wavefronts only help to fetch the partials
    if (redw[0] + redw[1] + redw[2] + redw[3] < 4.0e-8f) {
        // G2 = I + E with ||E||_F < 2e-4 (the usual case for a well-conditioned panel): the Cholesky factor is
        // I + X with X = strict_upper(E) + diag(E) / 2 and its inverse I - X, both up to O(||E||^2) < fp32 rounding.
#pragma unroll
        for (int q = 0; q < 16; ++q) {
            const int e = tid + NTHR * q;
            const int i = e >> 6, j = e & 63;
            const float g = B0[i * LS + j];
            const float x = (j > i) ? g : (j == i ? 0.5f * (g - 1.f) : 0.f);
            const float dg = (i == j) ? 1.f : 0.f;
            B0[i * LS + j] = (j >= i) ? dg + x : 0.f;
            B1[i * LS + j] = (j >= i) ? dg - x : 0.f;
        }
        __syncthreads();
    } else {
        chol_upper_64(B0, tid);                 // B0 = U2
        tri_inv_upper_64<false>(B0, B1, tid);   // B1 = U2^-1
    }
#pragma unroll
    for (int q = 0; q < 16; ++q) {
        const int e = tid + NTHR * q;
        B2[(e >> 6) * LS + (e & 63)] = u1r[q];
        B3[(e >> 6) * LS + (e & 63)] = q1r[q];
    }
    __syncthreads();
    // Rf = U2 U1 (upper x upper): kept in registers until the row signs are known;  Q_top = Q1_top U2^-1 -> B0
    f32x16 accR = zero16();
    if (qi <= qj) accR = lds_mma<0>(B0, B2, nullptr, qi, qj, 32 * qi, 32 * (qj + 1), lrow, lk);
    {
        const f32x16 accQ = lds_mma<0>(B3, B1, nullptr, qi, qj, 0, 32 * (qj + 1), lrow, lk);
        __syncthreads();                        // every wavefront has read U2 out of B0
        acc_to_lds(accQ, B0, qi, qj, lrow, lk);
    }
    __syncthreads();
    lu_signed_64(B0, sg, tid);                  // B0 = L \ U_lu, sg = S
    // V_top (the unit lower triangular L) to the panel; its transpose (unit upper triangular) to B3
#pragma unroll
    for (int q = 0; q < 16; ++q) {
        const int e = tid + NTHR * q;
        const int r = e >> 6, c = e & 63;
        if (c < r) A[(long)r * lda + c] = B0[r * LS + c];
        B3[r * LS + c] = (c > r) ? B0[c * LS + r] : (c == r ? 1.f : 0.f);
    }
    // both inverses in one sequence of barriers (its first barrier orders the writes of B3 before their reads):
    tri_inv_upper_64_pair<false, true>(B0, B2, B3, B4, tid);    // B2 = U_lu^-1, B4 = V_top^-T
    // Three products of upper triangular factors, kept in registers until the barrier below:
    //   Mm  = U2^-1 U_lu^-1,   T = -(U_lu S) V_top^-T,   Mm2 = Mm T = -(U2^-1 S) V_top^-T  (U_lu cancels)
    f32x16 accM = zero16(), accT = zero16(), acc2 = zero16();
    if (qi <= qj) {
        accM = lds_mma<0>(B1, B2, nullptr, qi, qj, 32 * qi, 32 * (qj + 1), lrow, lk);
        accT = lds_mma<1>(B0, B4, sg, qi, qj, 32 * qi, 32 * (qj + 1), lrow, lk);
        acc2 = lds_mma<0>(B1, B4, sg, qi, qj, 32 * qi, 32 * (qj + 1), lrow, lk);
    }
    {
        const int c = 32 * qj + lrow, rb = 32 * qi + 4 * lk;
        float sgr[16];                          // the signs of this thread's rows, requested together
#pragma unroll
        for (int v = 0; v < 16; ++v) sgr[v] = sg[rb + 8 * (v >> 2) + (v & 3)];
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int r = rb + 8 * (v >> 2) + (v & 3);
            const float t = (c >= r) ? -accT[v] : 0.f;
            Mm[r * B64 + c] = accM[v];
            Mm2[r * B64 + c] = -acc2[v];
            Tout[r * B64 + c] = t;
            B3[r * LS + c] = t;                 // nothing reads V_top^T any more
        }
        // the triangular factor S Rf: the whole quadrant right of the diagonal ones, the upper triangle of those
        float* Ar = A + (long)rb * lda + c;
        if (qi < qj) {
#pragma unroll
            for (int v = 0; v < 16; ++v) Ar[(long)(8 * (v >> 2) + (v & 3)) * lda] = sgr[v] * accR[v];
        } else if (qi == qj) {
#pragma unroll
            for (int v = 0; v < 16; ++v)
                if (c >= rb + 8 * (v >> 2) + (v & 3)) Ar[(long)(8 * (v >> 2) + (v & 3)) * lda] = sgr[v] * accR[v];
        }
    }
    __syncthreads();
    {   // Yp_top = V_top T (unit lower x upper)
        const int kq = qi < qj ? qi : qj;
        const f32x16 accY = lds_mma<2>(B0, B3, nullptr, qi, qj, 0, 32 * (kq + 1), lrow, lk);
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int r = 32 * qi + 8 * (v >> 2) + 4 * lk + (v & 3), c = 32 * qj + lrow;
            Yp[r * B64 + c] = accY[v];
        }
    }
}

__global__ __launch_bounds__(NSUM) void hr_finish_kernel(const float* __restrict__ part, int nparts, float* q1,
                                                         const float* __restrict__ U1, float* A, long lda, int m,
                                                         float* __restrict__ Tout, float* __restrict__ Yp,
                                                         float* __restrict__ Mm, float* __restrict__ Mm2,
                                                         float* __restrict__ tau, float* __restrict__ tslices,
                                                         unsigned* __restrict__ fb, unsigned* __restrict__ status,
                                                         unsigned long long* ready) {
    __builtin_amdgcn_s_setprio(3);   // the panel chain is latency-critical: win issue slots from co-resident GEMM waves
    if (threadIdx.x == 0) *ready = 0ull;   // "U1^-1 of the next panel is there": set by this panel's la_update_chol_kernel
    __shared__ float Bs[5 * B64 * LS];
    __shared__ float sg[B64];
    __shared__ float redw[4];
    hr_finish_body(part, nparts, q1, U1, A, lda, m, Tout, Yp, Mm, Mm2, tau, tslices, fb, status, Bs, sg, redw);
}


// ------------------------------------------------------------------------------------------------------------
// One launch per panel between consecutive tall panels: hr_finish_kernel, ts_mul_proj_kernel and
// la_update_chol_kernel as the phases of ONE kernel, for panels whose rows below the top block make one 128-row tile
// per workgroup.  What the two kernel boundaries ordered is ordered by three 8-byte words that only grow (agent-scope
// release / acquire, every poll bounded by the device clock; see HandOver):
//   ready1 = epoch    workgroup 0 has finished the panel's small step (Mm, Mm2, T, the top block, *fb are written);
//   count >= target   all nproj workgroups have written their rows of V and Yp and their partials of the projection and of
//                     C^T C (each adds 1; target = the sum over all launches so far, kept by the host);
//   ready2 = epoch    the extra workgroup has U1 and U1^-1 of the next panel;
//   rows >= target_rows   the workgroups below the top block have written their partials of C^T C (formed while workgroup
//                     0 works): the extra workgroup sums those ahead of time, off the chain of dependent steps.
// Workgroup 0: the small step, then the top 64 rows.  Workgroups 1 .. nproj - 1: one tile of rows each; while workgroup 0
// works they fetch their rows of Q1 and of the look-ahead columns C and form their part of C^T C; the rows of C stay in
// LDS through the update and the next panel's second step.  Workgroup nproj: the next panel's first small step, as in
// la_update_chol_kernel.  The nproj + 1 <= 34 workgroups run at the same time on 256 compute units; a poll that runs
// into its limit raises DQ_FLAG_SYNC_TIMEOUT and goes on, so every wavefront ends.
struct PanelSync {
    unsigned long long* ready1; unsigned long long* count; unsigned long long* ready2; unsigned long long* rows;
    unsigned long long epoch, target, target_rows;
    long long limit_ticks;
};

__device__ __forceinline__ void panel_wait(const unsigned long long* word, unsigned long long value, const PanelSync& ps,
                                           unsigned* status, int tid) {
    if (tid == 0) (void)handover_wait(word, value, ps.limit_ticks, status);
    __syncthreads();
}

// W2 = sum of the nproj projection partials -> Ws (row stride LS); NTHR threads, partials in groups of 8
__device__ __forceinline__ void sum_projection(const float* __restrict__ wpart, int nproj, float* Ws, int tid) {
    float4 s4[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) s4[q] = make_float4(0.f, 0.f, 0.f, 0.f);
    for (int z0 = 0; z0 < nproj; z0 += 8) {
        float4 t[4][8];
#pragma unroll
        for (int q = 0; q < 4; ++q)
#pragma unroll
            for (int z = 0; z < 8; ++z)
                t[q][z] = (z0 + z < nproj)
                              ? *reinterpret_cast<const float4*>(wpart + (long)(z0 + z) * B64 * B64 + 4 * (tid + NTHR * q))
                              : make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
        for (int q = 0; q < 4; ++q)
#pragma unroll
            for (int z = 0; z < 8; ++z) {
                s4[q].x += t[q][z].x; s4[q].y += t[q][z].y; s4[q].z += t[q][z].z; s4[q].w += t[q][z].w;
            }
    }
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const int e = 4 * (tid + NTHR * q);
        float* d = Ws + (e >> 6) * LS + (e & 63);
        d[0] = s4[q].x; d[1] = s4[q].y; d[2] = s4[q].z; d[3] = s4[q].w;
    }
}

constexpr int kFusedPool = 2 * RT * LS + 2 * B64 * B64;   // floats of LDS: two row tiles and two 64 x 64 matrices

__global__ __launch_bounds__(NSUM) void panel_fused_kernel(const float* part, int nparts, float* q1,
                                                           float* U1, float* U1inv, float* A, long lda, int m,
                                                           float* __restrict__ Tout, float* Yp, float* Mm, float* Mm2,
                                                           float* __restrict__ tau, float* __restrict__ tslices,
                                                           unsigned* fb, unsigned* status, float* wpart, float* gpart,
                                                           float* gearly, float* ctop, int nproj, PanelSync ps,
                                                           HandOver ho) {
    __builtin_amdgcn_s_setprio(3);
    __shared__ __attribute__((aligned(16))) float pool[kFusedPool];
    __shared__ float sg[B64];
    __shared__ float redw[4];
    static_assert(kFusedPool >= 5 * B64 * LS, "the small step's five matrices must fit the pool");
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int lrow = lane & 31, lk = lane >> 5;
    const int qi = (wave >> 1) & 1, qj = wave & 1;
    const int b = blockIdx.x;
    float* C = A + B64;
    float* Xs = pool;                       // a 128-row tile
    float* Cs = pool + RT * LS;             // a 128-row tile
    float* Ms = pool + 2 * RT * LS;         // 64 x 64, row stride 64
    float* Ms2 = Ms + B64 * B64;
    float* Ws = Ms;                         // 64 x 64, row stride LS (over Ms and the head of Ms2)

    if (b == nproj) {
        // ---- the next panel's U1 = chol(G), U1^-1 (see la_update_chol_kernel).  The partials of C^T C of the rows below
        // the top block are there long before the projections: summed now, while workgroup 0 still works
        panel_wait(ps.rows, ps.target_rows, ps, status, tid);
        constexpr int PERX = B64 * B64 / 4 / NSUM;
        float4 gsum[PERX];
        sum_partials_regs<NSUM, 16>(gearly + B64 * B64, nproj - 1, gsum, tid);
        panel_wait(ps.count, ps.target, ps, status, tid);
        float* S0 = pool;                   // V_top
        float* S1 = pool + B64 * LS;        // C_top, then C'_top
        float* Wx = pool + 2 * B64 * LS;
        float* Gs = pool + 3 * B64 * LS;
        float4 vt[4], ct[4];
        if (tid < NTHR) {
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int e = 4 * (tid + NTHR * q);
                vt[q] = *reinterpret_cast<const float4*>(A + (long)(e >> 6) * lda + (e & 63));
                ct[q] = *reinterpret_cast<const float4*>(ctop + e);
            }
        }
        {   // W2 = sum of the projection partials;  C^T C = the early sum + workgroup 0's part (the top rows)
            float4 wsum[PERX];
            sum_partials_regs<NSUM, 16, true>(wpart, nproj, wsum, tid);
#pragma unroll
            for (int q = 0; q < PERX; ++q) {
                const int e = 4 * (tid + NSUM * q);
                const bool upper = !((e >> 6) >= 32 && (e & 63) < 32);
                if (upper) {
                    const float4 t = *reinterpret_cast<const float4*>(gearly + e);
                    gsum[q].x += t.x; gsum[q].y += t.y; gsum[q].z += t.z; gsum[q].w += t.w;
                }
                float* dw = Wx + (e >> 6) * LS + (e & 63);
                float* dg = Gs + (e >> 6) * LS + (e & 63);
                dw[0] = wsum[q].x; dw[1] = wsum[q].y; dw[2] = wsum[q].z; dw[3] = wsum[q].w;
                dg[0] = gsum[q].x; dg[1] = gsum[q].y; dg[2] = gsum[q].z; dg[3] = gsum[q].w;
            }
            __syncthreads();
        }
        if (tid >= NTHR) return;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int e = 4 * (tid + NTHR * q);
            float* d0 = S0 + (e >> 6) * LS + (e & 63);
            float* d1 = S1 + (e >> 6) * LS + (e & 63);
            d0[0] = vt[q].x; d0[1] = vt[q].y; d0[2] = vt[q].z; d0[3] = vt[q].w;
            d1[0] = ct[q].x; d1[1] = ct[q].y; d1[2] = ct[q].z; d1[3] = ct[q].w;
        }
        __syncthreads();
        const f32x16 vw = lds_mma<2>(S0, Wx, nullptr, qi, qj, 0, B64, lrow, lk);   // V_top (unit lower) W2
        __syncthreads();
#pragma unroll
        for (int v = 0; v < 16; ++v) S1[(32 * qi + 8 * (v >> 2) + 4 * lk + (v & 3)) * LS + 32 * qj + lrow] -= vw[v];
        __syncthreads();
        if (qi <= qj) {
            f32x16 gt = zero16();
#pragma unroll 8
            for (int r = 0; r < B64; r += 2)
                gt = MFMA32(S1[(r + lk) * LS + 32 * qi + lrow], S1[(r + lk) * LS + 32 * qj + lrow], gt);
#pragma unroll
            for (int v = 0; v < 16; ++v) Gs[(32 * qi + 8 * (v >> 2) + 4 * lk + (v & 3)) * LS + 32 * qj + lrow] -= gt[v];
        }
        __syncthreads();
        chol_upper_64(Gs, tid);
        tri_inv_upper_64<false>(Gs, Wx, tid);
#pragma unroll
        for (int q = 0; q < 16; ++q) {
            const int e = tid + NTHR * q;
            U1[e] = Gs[(e >> 6) * LS + (e & 63)];
            U1inv[e] = Wx[(e >> 6) * LS + (e & 63)];
        }
        __syncthreads();
        if (tid == 0) handover_signal(ps.ready2, ps.epoch);
        return;
    }

    if (b == 0) {
        // ---- the panel's small step, then the top 64 rows
        hr_finish_body(part, nparts, q1, U1, A, lda, m, Tout, Yp, Mm, Mm2, tau, tslices, fb, status, pool, sg, redw);
        if (tid >= NTHR) return;
        __syncthreads();
        if (tid == 0) handover_signal(ps.ready1, ps.epoch);
        if (ho.wait_word != nullptr) {      // the look-ahead columns must have received the previous trailing update
            if (tid == 0) (void)handover_wait(ho.wait_word, ho.wait_value, (long long)ho.limit_us * 100, ho.flags);
            __syncthreads();
        }
        load_tile(Yp, B64, 0, B64, Xs, tid);
        load_tile(C, lda, 0, B64, Cs, tid);
        __syncthreads();
        f32x16 acc = zero16(), accg = zero16();
        proj_tile(Xs, Cs, acc, qi, qj, lrow, lk);
        gram_tile(Cs, accg, qi, qj, lrow, lk);
#pragma unroll
        for (int q = 0; q < 16; ++q) {
            const int e = tid + NTHR * q;
            ctop[e] = Cs[(e >> 6) * LS + (e & 63)];
        }
        store_partial(wpart, acc, qi, qj, lrow, lk);
        store_partial(gearly, accg, qi, qj, lrow, lk);
        __syncthreads();
        if (tid == 0) (void)__hip_atomic_fetch_add(ps.count, 1ull, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_AGENT);
        // the reflectors as stored, unit lower triangular, for the update of the top rows
        load_tile(A, lda, 0, B64, Xs, tid);
        __syncthreads();
        mask_unit_lower(Xs, tid);
        panel_wait(ps.count, ps.target, ps, status, tid);
        // the panel's reflectors and Yp are complete: the other streams may go on
        if (ho.signal_word != nullptr && tid == 0) handover_signal(ho.signal_word, ho.signal_value);
        sum_projection(wpart, nproj, Ws, tid);
        __syncthreads();
        f32x16 q0 = zero16(), q1v = zero16();
        mul_tile_full(Xs, Ws, q0, q1v, wave, lrow, lk);
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int r = 32 * wave + 8 * (v >> 2) + 4 * lk + (v & 3);
            if (r < B64) {
                C[(long)r * lda + lrow] = Cs[r * LS + lrow] - q0[v];
                C[(long)r * lda + 32 + lrow] = Cs[r * LS + 32 + lrow] - q1v[v];
            }
        }
        return;
    }

    // ---- one tile of rows below the top block
    if (tid >= NTHR) return;
    if (ho.wait_word != nullptr) {
        if (tid == 0) (void)handover_wait(ho.wait_word, ho.wait_value, (long long)ho.limit_us * 100, ho.flags);
        __syncthreads();
    }
    const int row0 = B64 + (b - 1) * RT;
    load_tile(q1, B64, row0, m, Xs, tid);
    load_tile(C, lda, row0, m, Cs, tid);
    __syncthreads();
    f32x16 accg = zero16();
    gram_tile(Cs, accg, qi, qj, lrow, lk);          // C_rows^T C_rows of the columns BEFORE the update
    store_partial(gearly + (long)b * B64 * B64, accg, qi, qj, lrow, lk);
    __syncthreads();
    if (tid == 0) (void)__hip_atomic_fetch_add(ps.rows, 1ull, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_AGENT);
    panel_wait(ps.ready1, ps.epoch, ps, status, tid);
    const bool fell_back = *fb != 0u;
    f32x16 v0 = zero16(), v1 = zero16();            // this wavefront's 32 rows of V
    if (!fell_back) {
        load_small64(Mm, Ms, tid);
        load_small64(Mm2, Ms2, tid);
        __syncthreads();
        mul_tile(Xs, Ms, v0, v1, wave, lrow, lk);
        f32x16 y0 = zero16(), y1 = zero16();
        mul_tile(Xs, Ms2, y0, y1, wave, lrow, lk);
        // each wavefront only read its own 32 rows of the tile: it may overwrite them with Yp right away
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int rl = 32 * wave + 8 * (v >> 2) + 4 * lk + (v & 3);
            Xs[rl * LS + lrow] = y0[v];
            Xs[rl * LS + 32 + lrow] = y1[v];
            if (row0 + rl < m) {
                A[(long)(row0 + rl) * lda + lrow] = v0[v];
                A[(long)(row0 + rl) * lda + 32 + lrow] = v1[v];
                Yp[(long)(row0 + rl) * B64 + lrow] = y0[v];
                Yp[(long)(row0 + rl) * B64 + 32 + lrow] = y1[v];
            }
        }
    } else {
        load_tile(Yp, B64, row0, m, Xs, tid);       // the fallback wrote V and Yp itself
    }
    __syncthreads();
    {
        f32x16 acc = zero16();
        proj_tile(Xs, Cs, acc, qi, qj, lrow, lk);
        store_partial(wpart + (long)b * B64 * B64, acc, qi, qj, lrow, lk);
    }
    __syncthreads();                                // every wavefront is done with Yp in Xs; all partials are stored
    if (tid == 0) (void)__hip_atomic_fetch_add(ps.count, 1ull, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_AGENT);
    if (!fell_back) {
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int rl = 32 * wave + 8 * (v >> 2) + 4 * lk + (v & 3);
            Xs[rl * LS + lrow] = v0[v];
            Xs[rl * LS + 32 + lrow] = v1[v];
        }
    } else {
        load_tile(A, lda, row0, m, Xs, tid);
    }
    panel_wait(ps.count, ps.target, ps, status, tid);
    sum_projection(wpart, nproj, Ws, tid);
    __syncthreads();
    {   // C_rows -= V_rows W2: to memory and, for the next panel's second step, kept in LDS
        f32x16 q0 = zero16(), q1v = zero16();
        mul_tile_full(Xs, Ws, q0, q1v, wave, lrow, lk);
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int rl = 32 * wave + 8 * (v >> 2) + 4 * lk + (v & 3);
            const float c0 = Cs[rl * LS + lrow] - q0[v], c1 = Cs[rl * LS + 32 + lrow] - q1v[v];
            Cs[rl * LS + lrow] = c0;
            Cs[rl * LS + 32 + lrow] = c1;
            if (row0 + rl < m) {
                C[(long)(row0 + rl) * lda + lrow] = c0;
                C[(long)(row0 + rl) * lda + 32 + lrow] = c1;
            }
        }
    }
    // ---- the next panel's second step for these rows: Q1 = C' U1^-1 and the partial of Q1^T Q1
    panel_wait(ps.ready2, ps.epoch, ps, status, tid);        // (its barrier also ends the reads of Ws)
    load_small64(U1inv, Ms, tid);
    __syncthreads();
    {
        f32x16 q0 = zero16(), q1v = zero16();
        mul_tile(Cs, Ms, q0, q1v, wave, lrow, lk);
        const int mn = m - B64, r0n = row0 - B64;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int rl = 32 * wave + 8 * (v >> 2) + 4 * lk + (v & 3);
            Cs[rl * LS + lrow] = q0[v];                      // own rows only, as above
            Cs[rl * LS + 32 + lrow] = q1v[v];
            if (r0n + rl < mn) {
                q1[(long)(r0n + rl) * B64 + lrow] = q0[v];
                q1[(long)(r0n + rl) * B64 + 32 + lrow] = q1v[v];
            }
        }
    }
    __syncthreads();
    f32x16 acc2 = zero16();
    gram_tile(Cs, acc2, qi, qj, lrow, lk);
    store_partial(gpart + (long)(b - 1) * B64 * B64, acc2, qi, qj, lrow, lk);
}

}  // namespace

size_t cholpanel_scratch_floats() { return (size_t)(3 * kCholMaxParts + 3) * B64 * B64 + 5 * B64 * B64 + 64; }

bool cholpanel_supported(const float* A, long lda, int m, int jb) {
    return jb == B64 && m >= B64 && m <= 8192 && (reinterpret_cast<uintptr_t>(A) & 15) == 0 && (lda & 3) == 0;
}

namespace {
struct TallScratch {
    float *part, *U1, *U1inv, *Mm, *Mm2, *ctop, *wpart, *gearly;
    unsigned* fb;
    unsigned long long* ready;
    explicit TallScratch(float* scratch) {
        part = scratch;                                            // kCholMaxParts + 1 Gram partials
        U1 = part + (size_t)(kCholMaxParts + 1) * B64 * B64;
        U1inv = U1 + B64 * B64;
        Mm = U1inv + B64 * B64;
        Mm2 = Mm + B64 * B64;
        ctop = Mm2 + B64 * B64;                                    // top block of the look-ahead columns before their update
        fb = reinterpret_cast<unsigned*>(ctop + B64 * B64);
        ready = reinterpret_cast<unsigned long long*>(ctop + B64 * B64 + 2);   // 8-byte aligned: the scratch is 256-byte aligned
        wpart = ctop + B64 * B64 + 64;                             // kCholMaxParts + 1 projection partials
        gearly = wpart + (size_t)(kCholMaxParts + 1) * B64 * B64;  // kCholMaxParts + 1 partials of C^T C (one-launch panels)
    }
};
// Row tiles of 128 per workgroup and number of workgroups (= Gram partials) for a panel of m rows.  More partials
// shorten the tall-skinny kernels but lengthen the one-workgroup sums; 32 was the knee at n = 4096 and 8192 (8: +20 %, 16: +5 %).
void tall_split(int m, int& tpw, int& nparts) {
    // 32 up to m = 4096, 64 above (30.4 against 31.0 ms for the QR at n = 8192)
    const int cap = m > 4096 ? 64 : 32;
    const int tiles = (m + RT - 1) / RT;
    tpw = (tiles + cap - 1) / cap;
    nparts = (tiles + tpw - 1) / tpw;
}
}  // namespace

hipError_t launch_cholqr_factor(float* A, long lda, int m, float* Tout, float* Yp, float* q1, float* scratch,
                                float* tau, float* tslices, unsigned* status, int have_gram, hipStream_t s) {
    if (!cholpanel_supported(A, lda, m, B64)) return hipErrorInvalidValue;
    const TallScratch ts(scratch);
    int tpw, nparts;
    tall_split(m, tpw, nparts);
    if (!have_gram) {   // otherwise the first two steps were done by the previous panel's launch_cholqr_finish
        hipLaunchKernelGGL(ts_gram_kernel, dim3(nparts), dim3(NTHR), 0, s, A, lda, m, tpw, ts.part);
        hipLaunchKernelGGL(chol_inv_kernel, dim3(1), dim3(NSUM), 0, s, ts.part, nparts, ts.U1, ts.U1inv);
        hipLaunchKernelGGL(ts_mul_gram_kernel, dim3(nparts), dim3(NTHR), 0, s, A, lda, m, tpw, ts.U1inv, q1, ts.part);
    }
    hipLaunchKernelGGL(hr_finish_kernel, dim3(1), dim3(NSUM), 0, s, ts.part, nparts, q1, ts.U1, A, lda, m, Tout, Yp,
                       ts.Mm, ts.Mm2, tau, tslices, ts.fb, status, ts.ready);
    return hipGetLastError();
}

hipError_t launch_cholqr_finish(float* A, long lda, int m, float* Yp, float* q1, float* scratch, int lookahead,
                                int next_gram, unsigned* status, hipStream_t s, const HandOver* ho) {
    const TallScratch ts(scratch);
    if (!lookahead) {
        if (ho != nullptr) return hipErrorInvalidValue;
        const int below = (m - B64 + RT - 1) / RT;   // a square last panel has no rows below its top block
        if (below > 0)
            hipLaunchKernelGGL(ts_mul_kernel, dim3(below), dim3(NTHR), 0, s, q1, m, B64, ts.Mm, ts.Mm2, A, lda, Yp, ts.fb);
        return hipGetLastError();
    }
    // the rows below the top block are split exactly as the next panel (m - 64 rows) splits its own rows
    int tpw, nparts;
    tall_split(m - B64, tpw, nparts);
    const HandOver h = ho != nullptr ? *ho : HandOver();
    float* gpart = next_gram ? ts.part : static_cast<float*>(nullptr);
    hipLaunchKernelGGL(ts_mul_proj_kernel, dim3(nparts + 1), dim3(NTHR), 0, s, q1, m, ts.Mm, ts.Mm2, A, lda, Yp, ts.fb,
                       tpw, ts.wpart, gpart, ts.ctop, h);
    // The extra workgroup is the longest one: with NSUM threads its two sums take 3 batches of loads each instead of 5
    // (n = 4096: 7.15 -> 7.01 ms for the QR); above 4096 rows, where the kernel has twice the workgroups and the chain
    // is not what bounds the QR, the wider workgroups cost more than they give (n = 8192: 27.95 -> 28.45 ms).
    const bool wide = m <= 4096;
    if (wide)
        hipLaunchKernelGGL(la_update_chol_kernel<NSUM>, dim3(nparts + 1 + (next_gram ? 1 : 0)), dim3(NSUM), 0, s, A, lda, m,
                           ts.wpart, nparts + 1, tpw, gpart, ts.ctop, ts.U1, ts.U1inv, q1, ts.ready, status, h);
    else
        hipLaunchKernelGGL(la_update_chol_kernel<NTHR>, dim3(nparts + 1 + (next_gram ? 1 : 0)), dim3(NTHR), 0, s, A, lda, m,
                           ts.wpart, nparts + 1, tpw, gpart, ts.ctop, ts.U1, ts.U1inv, q1, ts.ready, status, h);
    return hipGetLastError();
}

int cholqr_fused_workgroups(int m) {
    int tpw, nparts;
    tall_split(m - B64, tpw, nparts);
    return tpw == 1 ? nparts + 1 : 0;
}

hipError_t launch_cholqr_fused(float* A, long lda, int m, float* Tout, float* Yp, float* q1, float* scratch, float* tau,
                               float* tslices, unsigned* status, unsigned long long* words, unsigned long long epoch,
                               unsigned long long target, unsigned long long target_rows, long limit_us, hipStream_t s,
                               const HandOver* ho) {
    if (!cholpanel_supported(A, lda, m, B64) || m < 2 * B64) return hipErrorInvalidValue;
    const int nproj = cholqr_fused_workgroups(m);
    if (nproj < 2 || nproj > kCholMaxParts + 1) return hipErrorInvalidValue;
    const TallScratch ts(scratch);
    int tpw, nparts;
    tall_split(m, tpw, nparts);          // the partials of Q1^T Q1 that the previous panel's kernels left
    PanelSync ps;
    ps.ready1 = words; ps.count = words + 1; ps.ready2 = words + 2; ps.rows = words + 3;
    ps.epoch = epoch; ps.target = target; ps.target_rows = target_rows; ps.limit_ticks = (long long)limit_us * 100;
    const HandOver h = ho != nullptr ? *ho : HandOver();
    hipLaunchKernelGGL(panel_fused_kernel, dim3(nproj + 1), dim3(NSUM), 0, s, ts.part, nparts, q1, ts.U1, ts.U1inv, A, lda,
                       m, Tout, Yp, ts.Mm, ts.Mm2, tau, tslices, ts.fb, status, ts.wpart, ts.part, ts.gearly, ts.ctop, nproj, ps, h);
    return hipGetLastError();
}

}  // namespace dq
