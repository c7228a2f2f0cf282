// 64 x 64 dense building blocks that live in LDS and run on one workgroup of 256 threads (4 wavefronts):
// products on the fp32 matrix cores and the inverse of a triangular matrix.  Used by the tall-panel route of the
// QR (Alg. 2 in blocked form) and by the triangular solve of the derivative through the QR (the last step of Alg. 1).
// Matrices are row-major with row stride LS; every routine that says so ends with a workgroup barrier and must
// be called by all 256 threads.
#pragma once

#include "dq_internal.h"

namespace dq {

typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int B64 = 64;          // matrix size handled here (= the QR panel width)
constexpr int LS = 65;           // LDS row stride (conflict-free column walks)
constexpr int NTHR = 256;        // threads per workgroup (4 wavefronts)

#define MFMA32(a, b, c) __builtin_amdgcn_mfma_f32_32x32x2f32((a), (b), (c), 0, 0, 0)

__device__ __forceinline__ f32x16 zero16() {
    f32x16 z;
#pragma unroll
    for (int v = 0; v < 16; ++v) z[v] = 0.f;
    return z;
}

// One level of the triangular-inverse merge for diagonal blocks of size BL (8 or 16), see tri_inv_upper_64.
template <int BL>
__device__ __forceinline__ void tri_inv_level(const float* U, float* X, int tid) {
    constexpr int PER_PAIR = BL * BL;
    constexpr int TOTAL = (B64 / (2 * BL)) * PER_PAIR;
    constexpr int ITERS = (TOTAL + NTHR - 1) / NTHR;
    float acc[ITERS];
#pragma unroll
    for (int it = 0; it < ITERS; ++it) {                   // scratch (lower-left block of the pair) = B C^-1
        const int e = tid + NTHR * it;
        const int o = (e / PER_PAIR) * 2 * BL, r = e % PER_PAIR;
        const int i = r / BL, j = r % BL;
        float t = 0.f;
#pragma unroll 4
        for (int k = 0; k < BL; ++k) t += U[(o + i) * LS + o + BL + k] * X[(o + BL + k) * LS + o + BL + j];
        acc[it] = t;
    }
#pragma unroll
    for (int it = 0; it < ITERS; ++it) {
        const int e = tid + NTHR * it;
        const int o = (e / PER_PAIR) * 2 * BL, r = e % PER_PAIR;
        if (e < TOTAL) X[(o + BL + r / BL) * LS + o + r % BL] = acc[it];
    }
    __syncthreads();
#pragma unroll
    for (int it = 0; it < ITERS; ++it) {                   // X12 = -A^-1 scratch
        const int e = tid + NTHR * it;
        const int o = (e / PER_PAIR) * 2 * BL, r = e % PER_PAIR;
        const int i = r / BL, j = r % BL;
        float t = 0.f;
#pragma unroll 4
        for (int k = 0; k < BL; ++k) t += X[(o + i) * LS + o + k] * X[(o + BL + k) * LS + o + j];
        acc[it] = t;
    }
    __syncthreads();
#pragma unroll
    for (int it = 0; it < ITERS; ++it) {
        const int e = tid + NTHR * it;
        const int o = (e / PER_PAIR) * 2 * BL, r = e % PER_PAIR;
        if (e < TOTAL) {
            X[(o + r / BL) * LS + o + BL + r % BL] = -acc[it];
            X[(o + BL + r / BL) * LS + o + r % BL] = 0.f;
        }
    }
    __syncthreads();
}

// X = inverse of the upper-triangular matrix held in the upper triangle of U (what lies below U's diagonal is
// ignored); X's strict lower triangle is zero on return.  8 x 8 diagonal blocks by substitution, then neighbours are
// merged level by level:  inv [[A, B], [0, C]] = [[A^-1, -A^-1 B C^-1], [0, C^-1]], the last level on the matrix
// cores.  The lower-left block of each merged pair is used as scratch for B C^-1 and cleared afterwards.
// UNIT: the diagonal of U is taken as 1.
template <bool UNIT>
__device__ __forceinline__ void tri_inv_upper_64(const float* U, float* X, int tid) {
    const int lane = tid & 63, wave = tid >> 6, lrow = lane & 31, lk = lane >> 5;
#pragma unroll
    for (int q = 0; q < 16; ++q) {
        const int e = tid + NTHR * q;
        X[(e >> 6) * LS + (e & 63)] = 0.f;
    }
    __syncthreads();
    if (tid < 64) {
        const int o = 8 * (tid >> 3), c = tid & 7;
        float u[8][8], x[8], ru[8];
#pragma unroll
        for (int r = 0; r < 8; ++r)
#pragma unroll
            for (int q = r; q < 8; ++q) u[r][q] = U[(o + r) * LS + o + q];
#pragma unroll
        for (int r = 0; r < 8; ++r) ru[r] = UNIT ? 1.f : __builtin_amdgcn_rcpf(u[r][r]);   // hardware reciprocal (1 ulp)
#pragma unroll
        for (int r = 7; r >= 0; --r) {
            float t = (r == c) ? 1.f : 0.f;
#pragma unroll
            for (int q = r + 1; q < 8; ++q) t -= u[r][q] * x[q];
            x[r] = t * ru[r];
        }
#pragma unroll
        for (int r = 0; r < 8; ++r) X[(o + r) * LS + o + c] = x[r];
    }
    __syncthreads();
    tri_inv_level<8>(U, X, tid);
    tri_inv_level<16>(U, X, tid);
    if (wave == 0) {                                       // scratch (rows 32.., cols 0..31) = U12 C^-1
        f32x16 acc = zero16();
#pragma unroll
        for (int kk = 0; kk < 32; kk += 2)
            acc = MFMA32(U[lrow * LS + 32 + kk + lk], X[(32 + kk + lk) * LS + 32 + lrow], acc);
#pragma unroll
        for (int v = 0; v < 16; ++v) X[(32 + 8 * (v >> 2) + 4 * lk + (v & 3)) * LS + lrow] = acc[v];
    }
    __syncthreads();
    if (wave == 0) {
        f32x16 acc = zero16();
#pragma unroll
        for (int kk = 0; kk < 32; kk += 2)
            acc = MFMA32(X[lrow * LS + kk + lk], X[(32 + kk + lk) * LS + lrow], acc);
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int r = 8 * (v >> 2) + 4 * lk + (v & 3);
            X[r * LS + 32 + lrow] = -acc[v];
        }
        // the reads of the scratch block above are complete (their results fed the products): clear it
#pragma unroll
        for (int v = 0; v < 16; ++v) X[(32 + 8 * (v >> 2) + 4 * lk + (v & 3)) * LS + lrow] = 0.f;
    }
    __syncthreads();
}

// Two independent inverses in the same sequence of barriers (the routine is bound by its dozen barriers, not by its
// arithmetic): X0 = inv(U0), X1 = inv(U1), each as tri_inv_upper_64 computes it, UNIT0 / UNIT1 as UNIT there.
template <int BL>
__device__ __forceinline__ void tri_inv_level_pair(const float* U0, float* X0, const float* U1, float* X1, int tid) {
    constexpr int PER_PAIR = BL * BL;
    constexpr int TOTAL = (B64 / (2 * BL)) * PER_PAIR;
    constexpr int ITERS = (TOTAL + NTHR - 1) / NTHR;
    float acc[2][ITERS];
#pragma unroll
    for (int s = 0; s < 2; ++s) {
        const float* U = s ? U1 : U0;
        const float* X = s ? X1 : X0;
#pragma unroll
        for (int it = 0; it < ITERS; ++it) {               // scratch (lower-left block of the pair) = B C^-1
            const int e = tid + NTHR * it;
            const int o = (e / PER_PAIR) * 2 * BL, r = e % PER_PAIR;
            const int i = r / BL, j = r % BL;
            float t = 0.f;
#pragma unroll 4
            for (int k = 0; k < BL; ++k) t += U[(o + i) * LS + o + BL + k] * X[(o + BL + k) * LS + o + BL + j];
            acc[s][it] = t;
        }
    }
#pragma unroll
    for (int s = 0; s < 2; ++s) {
        float* X = s ? X1 : X0;
#pragma unroll
        for (int it = 0; it < ITERS; ++it) {
            const int e = tid + NTHR * it;
            const int o = (e / PER_PAIR) * 2 * BL, r = e % PER_PAIR;
            if (e < TOTAL) X[(o + BL + r / BL) * LS + o + r % BL] = acc[s][it];
        }
    }
    __syncthreads();
#pragma unroll
    for (int s = 0; s < 2; ++s) {
        const float* X = s ? X1 : X0;
#pragma unroll
        for (int it = 0; it < ITERS; ++it) {               // X12 = -A^-1 scratch
            const int e = tid + NTHR * it;
            const int o = (e / PER_PAIR) * 2 * BL, r = e % PER_PAIR;
            const int i = r / BL, j = r % BL;
            float t = 0.f;
#pragma unroll 4
            for (int k = 0; k < BL; ++k) t += X[(o + i) * LS + o + k] * X[(o + BL + k) * LS + o + j];
            acc[s][it] = t;
        }
    }
    __syncthreads();
#pragma unroll
    for (int s = 0; s < 2; ++s) {
        float* X = s ? X1 : X0;
#pragma unroll
        for (int it = 0; it < ITERS; ++it) {
            const int e = tid + NTHR * it;
            const int o = (e / PER_PAIR) * 2 * BL, r = e % PER_PAIR;
            if (e < TOTAL) {
                X[(o + r / BL) * LS + o + BL + r % BL] = -acc[s][it];
                X[(o + BL + r / BL) * LS + o + r % BL] = 0.f;
            }
        }
    }
    __syncthreads();
}

template <bool UNIT0, bool UNIT1>
__device__ __forceinline__ void tri_inv_upper_64_pair(const float* U0, float* X0, const float* U1, float* X1, int tid) {
    const int lane = tid & 63, wave = tid >> 6, lrow = lane & 31, lk = lane >> 5;
#pragma unroll
    for (int q = 0; q < 16; ++q) {
        const int e = tid + NTHR * q;
        X0[(e >> 6) * LS + (e & 63)] = 0.f;
        X1[(e >> 6) * LS + (e & 63)] = 0.f;
    }
    __syncthreads();
    if (tid < 128) {                                       // 8 x 8 diagonal blocks: wavefront 0 those of U0, wavefront 1 those of U1
        const bool second = tid >= 64;
        const float* U = second ? U1 : U0;
        float* X = second ? X1 : X0;
        const bool unit = second ? UNIT1 : UNIT0;
        const int t64 = tid & 63;
        const int o = 8 * (t64 >> 3), c = t64 & 7;
        float u[8][8], x[8], ru[8];
#pragma unroll
        for (int r = 0; r < 8; ++r)
#pragma unroll
            for (int q = r; q < 8; ++q) u[r][q] = U[(o + r) * LS + o + q];
#pragma unroll
        for (int r = 0; r < 8; ++r) ru[r] = unit ? 1.f : __builtin_amdgcn_rcpf(u[r][r]);   // hardware reciprocal (1 ulp)
#pragma unroll
        for (int r = 7; r >= 0; --r) {
            float t = (r == c) ? 1.f : 0.f;
#pragma unroll
            for (int q = r + 1; q < 8; ++q) t -= u[r][q] * x[q];
            x[r] = t * ru[r];
        }
#pragma unroll
        for (int r = 0; r < 8; ++r) X[(o + r) * LS + o + c] = x[r];
    }
    __syncthreads();
    tri_inv_level_pair<8>(U0, X0, U1, X1, tid);
    tri_inv_level_pair<16>(U0, X0, U1, X1, tid);
    const float* U = wave == 1 ? U1 : U0;
    float* X = wave == 1 ? X1 : X0;
    if (wave < 2) {                                        // scratch (rows 32.., cols 0..31) = U12 C^-1
        f32x16 acc = zero16();
#pragma unroll
        for (int kk = 0; kk < 32; kk += 2)
            acc = MFMA32(U[lrow * LS + 32 + kk + lk], X[(32 + kk + lk) * LS + 32 + lrow], acc);
#pragma unroll
        for (int v = 0; v < 16; ++v) X[(32 + 8 * (v >> 2) + 4 * lk + (v & 3)) * LS + lrow] = acc[v];
    }
    __syncthreads();
    if (wave < 2) {
        f32x16 acc = zero16();
#pragma unroll
        for (int kk = 0; kk < 32; kk += 2)
            acc = MFMA32(X[lrow * LS + kk + lk], X[(32 + kk + lk) * LS + lrow], acc);
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int r = 8 * (v >> 2) + 4 * lk + (v & 3);
            X[r * LS + 32 + lrow] = -acc[v];
        }
        // the reads of the scratch block above are complete (their results fed the products): clear it
#pragma unroll
        for (int v = 0; v < 16; ++v) X[(32 + 8 * (v >> 2) + 4 * lk + (v & 3)) * LS + lrow] = 0.f;
    }
    __syncthreads();
}

// This wavefront's 32 x 32 quadrant (qi, qj) of  A diag(kscale) B  over k in [klo, khi) (multiples of 32, at most 64
// apart), both operands in LDS.  AMODE 1: entries of A below its diagonal are taken as zero; AMODE 2: A is taken as unit
// lower triangular (stored diagonal and upper part ignored); AMODE 0: as stored.
// All operands of a product are requested before its first matrix-core instruction: a single wavefront per SIMD has
// nothing else to hide the LDS latency with, and the compiler otherwise waits for every pair of operands in turn.
template <int AMODE, bool SCALE>
__device__ __forceinline__ void lds_mma_fetch(const float* A, const float* Bm, const float* kscale, int row, int col,
                                              int k0, int lk, float (&a)[16], float (&b)[16]) {
#pragma unroll
    for (int u = 0; u < 16; ++u) {
        const int k = k0 + 2 * u + lk;
        a[u] = A[row * LS + k];
        b[u] = Bm[k * LS + col];
    }
    if (SCALE) {
        float s[16];
#pragma unroll
        for (int u = 0; u < 16; ++u) s[u] = kscale[k0 + 2 * u + lk];
#pragma unroll
        for (int u = 0; u < 16; ++u) {
            const int k = k0 + 2 * u + lk;
            if (AMODE == 1 && k < row) a[u] = 0.f;
            if (AMODE == 2) a[u] = (k < row) ? a[u] : (k == row ? 1.f : 0.f);
            a[u] *= s[u];
        }
    } else {
#pragma unroll
        for (int u = 0; u < 16; ++u) {
            const int k = k0 + 2 * u + lk;
            if (AMODE == 1 && k < row) a[u] = 0.f;
            if (AMODE == 2) a[u] = (k < row) ? a[u] : (k == row ? 1.f : 0.f);
        }
    }
}

template <int AMODE>
__device__ __forceinline__ f32x16 lds_mma(const float* A, const float* Bm, const float* kscale, int qi, int qj,
                                          int klo, int khi, int lrow, int lk) {
    f32x16 acc = zero16();
    if (khi <= klo) return acc;
    const int row = 32 * qi + lrow, col = 32 * qj + lrow;
    const bool two = khi - klo > 32;                      // the same for every lane of the wavefront
    float a0[16], b0[16], a1[16], b1[16];
    if (kscale != nullptr) {
        lds_mma_fetch<AMODE, true>(A, Bm, kscale, row, col, klo, lk, a0, b0);
        if (two) lds_mma_fetch<AMODE, true>(A, Bm, kscale, row, col, klo + 32, lk, a1, b1);
    } else {
        lds_mma_fetch<AMODE, false>(A, Bm, kscale, row, col, klo, lk, a0, b0);
        if (two) lds_mma_fetch<AMODE, false>(A, Bm, kscale, row, col, klo + 32, lk, a1, b1);
    }
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int u = 0; u < 16; ++u) acc = MFMA32(a0[u], b0[u], acc);
    if (two) {
#pragma unroll
        for (int u = 0; u < 16; ++u) acc = MFMA32(a1[u], b1[u], acc);
    }
    return acc;
}

__device__ __forceinline__ void acc_to_lds(const f32x16& acc, float* Bm, int qi, int qj, int lrow, int lk) {
#pragma unroll
    for (int v = 0; v < 16; ++v) Bm[(32 * qi + 8 * (v >> 2) + 4 * lk + (v & 3)) * LS + 32 * qj + lrow] = acc[v];
}

}  // namespace dq
