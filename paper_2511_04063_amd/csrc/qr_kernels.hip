// Blocked Householder QR pieces (Alg. 2 of the paper's appendix, in LAPACK-style compact-WY form):
//   * the panel factorisation (one workgroup, panel columns held in registers slice by slice),
//   * the triangular T factor of a panel's block reflector  H_1 ... H_jb = I - V T V^T,
//   * sign normalisation diag(U) >= 0 (the reading that makes R of Sec. 4.3 unique), and small helpers.
//
// Reflector convention: H = I - tau v v^T with v[0] = 1 implied, beta = -sign(alpha) ||x||,
// tau = (beta - alpha) / beta, v[1:] = x[1:] / (alpha - beta).  This is the same reflection as Alg. 2's
// normalised v = x + sign(x_1)||x|| e_1 (H = I - 2 v v^T / v^T v), stored without the normalisation.
#include "dq_internal.h"
#include "dq_wave.h"
#include "qr_panel_body.h"

namespace dq {
namespace {

template <int NT, int Q, int SW, int VCH>
__global__ __launch_bounds__(NT) void qr_panel_kernel(float* __restrict__ A, long lda, int m, int jb,
                                                      float* __restrict__ tau, float* Vs, float* __restrict__ tslices,
                                                      unsigned* flags, int vec) {
    qr_panel_body<NT, Q, SW, VCH>(A, lda, m, jb, tau, Vs, tslices, flags, vec);
}

__global__ __launch_bounds__(256) void unpack_reflectors_kernel(float* __restrict__ A, long lda, int m, int jb,
                                                                const float* __restrict__ Vs, int mp, int sw, int vec) {
    unpack_reflectors_body(A, lda, m, jb, Vs, mp, sw, vec, (long)blockIdx.x * 256 + threadIdx.x, (long)gridDim.x * 256);
}

// T factor of a panel's block reflector  H_1 ... H_jb = I - V T V^T  from the T factors of its column slices
// (sw x sw each, from the panel kernel) and the Gram matrix G = V^T V, by merging neighbours level by level:
//   T = [[T1, -T1 (V1^T V2) T2], [0, T2]].
// The input is the split-K partials of V^T [V | C] (jb x (jb + nla)); the kernel sums them, builds T and also
// returns W2 = T^T (V^T C) (jb x nla, leading dimension kPanel) for the update of the nla look-ahead columns.
__global__ __launch_bounds__(1024) void tfactor_kernel(const float* __restrict__ gpart, int splits, long stride,
                                                       long ldp, int jb, int nla, const float* __restrict__ tslices,
                                                       int sw, float* __restrict__ Tout, float* __restrict__ W2out) {
    typedef float f32x16 __attribute__((ext_vector_type(16)));
    __shared__ float Gs[kPanel][kPanel + 1];
    __shared__ float Ts[kPanel][kPanel + 1];
    __shared__ float Xs[kPanel][kPanel + 1];
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int lrow = lane & 31, lk = lane >> 5;
    float wreg[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const int e = tid + 1024 * q;
        const int i = e / kPanel, j = e % kPanel;
        float t = 0.f, w = 0.f;
        // up to 16 partials, all loads issued before the sums (the caller limits the split count to 16)
        float pt[16], pw[16];
#pragma unroll
        for (int z = 0; z < 16; ++z) {
            pt[z] = (z < splits && i < jb && j < jb) ? gpart[(long)z * stride + (long)i * ldp + j] : 0.f;
            pw[z] = (z < splits && i < jb && j < nla) ? gpart[(long)z * stride + (long)i * ldp + jb + j] : 0.f;
        }
#pragma unroll
        for (int z = 0; z < 16; ++z) { t += pt[z]; w += pw[z]; }
        wreg[q] = w;
        Gs[i][j] = t;
        float tv = 0.f;
        if (i / sw == j / sw && i < jb && j < jb) tv = tslices[(i / sw) * sw * sw + (i % sw) * sw + (j % sw)];
        Ts[i][j] = tv;
    }
    __syncthreads();
    // levels below 32: plain loops (a few hundred short dot products)
    for (int b = sw; b < 32; b <<= 1) {
        const int per_pair = b * b;
        const int total = (kPanel / (2 * b)) * per_pair;
        for (int e = tid; e < total; e += 1024) {          // X = G12 * T2
            const int o = (e / per_pair) * 2 * b, r = e % per_pair;
            const int i = r / b, j = r % b;
            float acc = 0.f;
            for (int k = 0; k <= j; ++k) acc += Gs[o + i][o + b + k] * Ts[o + b + k][o + b + j];
            Xs[o + i][o + b + j] = acc;
        }
        __syncthreads();
        for (int e = tid; e < total; e += 1024) {          // T12 = -T1 * X
            const int o = (e / per_pair) * 2 * b, r = e % per_pair;
            const int i = r / b, j = r % b;
            float acc = 0.f;
            for (int k = i; k < b; ++k) acc += Ts[o + i][o + k] * Xs[o + k][o + b + j];
            Ts[o + i][o + b + j] = -acc;
        }
        __syncthreads();
    }
    // level 32 -> 64 on the matrix cores (one wavefront, two 32 x 32 x 32 products):
    //   X = G[0:32, 32:64] * T[32:64, 32:64],   T[0:32, 32:64] = -T[0:32, 0:32] * X
    if (wave == 0) {
        f32x16 acc;
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[v] = 0.f;
#pragma unroll
        for (int kk = 0; kk < 32; kk += 2)
            acc = __builtin_amdgcn_mfma_f32_32x32x2f32(Gs[lrow][32 + kk + lk], Ts[32 + kk + lk][32 + lrow], acc, 0, 0, 0);
#pragma unroll
        for (int v = 0; v < 16; ++v) Xs[8 * (v >> 2) + 4 * lk + (v & 3)][32 + lrow] = acc[v];
    }
    __syncthreads();
    if (wave == 0) {
        f32x16 acc;
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[v] = 0.f;
#pragma unroll
        for (int kk = 0; kk < 32; kk += 2)
            acc = __builtin_amdgcn_mfma_f32_32x32x2f32(Ts[lrow][kk + lk], Xs[kk + lk][32 + lrow], acc, 0, 0, 0);
#pragma unroll
        for (int v = 0; v < 16; ++v) Ts[8 * (v >> 2) + 4 * lk + (v & 3)][32 + lrow] = -acc[v];
    }
    __syncthreads();
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const int e = tid + 1024 * q;
        Tout[e] = Ts[e / kPanel][e % kPanel];
        Gs[e / kPanel][e % kPanel] = wreg[q];           // G is no longer needed: keep W = V^T C there
    }
    __syncthreads();
    // W2 = T^T W (64 x 64 x 64) on the matrix cores: wavefronts 0..3 take one 32 x 32 tile each.
    // A operand: (T^T)[m][k] = Ts[k][m];  B operand: W[k][n] = Gs[k][n].
    if (nla > 0 && wave < 4) {
        const int m0 = (wave >> 1) * 32, n0 = (wave & 1) * 32;
        f32x16 acc;
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[v] = 0.f;
#pragma unroll
        for (int kk = 0; kk < kPanel; kk += 2)
            acc = __builtin_amdgcn_mfma_f32_32x32x2f32(Ts[kk + lk][m0 + lrow], Gs[kk + lk][n0 + lrow], acc, 0, 0, 0);
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int r = m0 + 8 * (v >> 2) + 4 * lk + (v & 3), cc = n0 + lrow;
            if (r < jb && cc < nla) W2out[r * kPanel + cc] = acc[v];
        }
    }
}

__global__ __launch_bounds__(256) void copy2d_kernel(const float* __restrict__ src, long lds, float* __restrict__ dst,
                                                     long ldd, int rows, int cols) {
    const long total = (long)rows * cols;
    for (long e = (long)blockIdx.x * 256 + threadIdx.x; e < total; e += (long)gridDim.x * 256) {
        const int r = (int)(e / cols), c = (int)(e % cols);
        dst[(long)r * ldd + c] = (src != nullptr) ? src[(long)r * lds + c] : 0.f;
    }
}

// The two kernels above with 16-byte accesses and 32-bit index arithmetic (cols a multiple of 4, 16-byte aligned rows,
// fewer than 2^31 pieces).
__global__ __launch_bounds__(256) void copy2d_vec_kernel(const float* __restrict__ src, long lds, float* __restrict__ dst,
                                                         long ldd, unsigned total4, unsigned cols4) {
    for (unsigned e = blockIdx.x * 256u + threadIdx.x; e < total4; e += gridDim.x * 256u) {
        const unsigned r = e / cols4, c = (e - r * cols4) << 2;
        float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
        if (src != nullptr) v = *reinterpret_cast<const float4*>(src + (long)r * lds + c);
        *reinterpret_cast<float4*>(dst + (long)r * ldd + c) = v;
    }
}
__global__ __launch_bounds__(256) void identity_vec_kernel(float* __restrict__ A, long lda, unsigned total4, unsigned cols4) {
    for (unsigned e = blockIdx.x * 256u + threadIdx.x; e < total4; e += gridDim.x * 256u) {
        const unsigned r = e / cols4, c = (e - r * cols4) << 2;
        *reinterpret_cast<float4*>(A + (long)r * lda + c) =
            make_float4(r == c ? 1.f : 0.f, r == c + 1 ? 1.f : 0.f, r == c + 2 ? 1.f : 0.f, r == c + 3 ? 1.f : 0.f);
    }
}

__global__ __launch_bounds__(256) void identity_kernel(float* __restrict__ A, long lda, int n) {
    const long total = (long)n * n;
    for (long e = (long)blockIdx.x * 256 + threadIdx.x; e < total; e += (long)gridDim.x * 256) {
        const int r = (int)(e / n), c = (int)(e % n);
        A[(long)r * lda + c] = (r == c) ? 1.f : 0.f;
    }
}

__global__ __launch_bounds__(256) void fill_u32_kernel(unsigned* p, long count, unsigned v) {
    for (long e = (long)blockIdx.x * 256 + threadIdx.x; e < count; e += (long)gridDim.x * 256) p[e] = v;
}

// The same with 16-byte accesses (n, leading dimensions multiples of 4, 16-byte aligned bases): a workgroup owns a strip
// of 1024 columns for kSignRows rows; a thread reads the four diagonal entries that give its column signs once (the only
// scattered loads), the row sign is uniform.  Pieces of A wholly below the diagonal are not read.
constexpr int kSignRows = 32;
__global__ __launch_bounds__(256) void sign_normalise_vec_kernel(const float* __restrict__ Afac, long lda, int n,
                                                                 float* __restrict__ R, long ldr, float* __restrict__ U,
                                                                 long ldu, unsigned* flags) {
    const int c = (blockIdx.x * 256 + threadIdx.x) * 4;
    if (c >= n) return;
    const int r0 = blockIdx.y * kSignRows;
    const int r1 = (r0 + kSignRows < n) ? r0 + kSignRows : n;
    float sc[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const float d = Afac[(long)(c + q) * lda + c + q];
        sc[q] = d >= 0.f ? 1.f : -1.f;
        if (blockIdx.y == 0) {
            if (!(fabsf(d) <= 3.0e38f)) atomicOr(flags, DQ_FLAG_NONFINITE);
            else if (d == 0.f) atomicOr(flags, DQ_FLAG_SINGULAR);
        }
    }
    // eight rows at a time, every load of the eight before the first store (R is updated in place: a load behind a store
    // to the same array waits for it, and row by row the strip would take one trip to memory per row)
    constexpr int G = 8;
    static_assert(kSignRows % G == 0, "whole groups of rows");
    for (int rg = r0; rg < r1; rg += G) {
        float4 v[G], a[G];
        float sr[G];
#pragma unroll
        for (int i = 0; i < G; ++i) {
            const int r = rg + i;
            v[i] = make_float4(0.f, 0.f, 0.f, 0.f); a[i] = v[i]; sr[i] = 1.f;
            if (r < r1) {
                v[i] = *reinterpret_cast<const float4*>(R + (long)r * ldr + c);
                if (U != nullptr && c + 3 >= r) {
                    sr[i] = Afac[(long)r * lda + r] >= 0.f ? 1.f : -1.f;
                    a[i] = *reinterpret_cast<const float4*>(Afac + (long)r * lda + c);
                }
            }
        }
#pragma unroll
        for (int i = 0; i < G; ++i) {
            const int r = rg + i;
            if (r < r1) {
                float4 w = v[i];
                w.x *= sc[0]; w.y *= sc[1]; w.z *= sc[2]; w.w *= sc[3];
                *reinterpret_cast<float4*>(R + (long)r * ldr + c) = w;
                if (U != nullptr) {
                    float4 u = make_float4(0.f, 0.f, 0.f, 0.f);
                    if (c + 3 >= r) {
                        u.x = c >= r ? sr[i] * a[i].x : 0.f;
                        u.y = c + 1 >= r ? sr[i] * a[i].y : 0.f;
                        u.z = c + 2 >= r ? sr[i] * a[i].z : 0.f;
                        u.w = c + 3 >= r ? sr[i] * a[i].w : 0.f;
                    }
                    *reinterpret_cast<float4*>(U + (long)r * ldu + c) = u;
                }
            }
        }
    }
}

// s_j = +1 if Afac[j][j] >= 0 else -1;  R[:, j] *= s_j;  U[i][j] = s_i * Afac[i][j] for j >= i, else 0.
__global__ __launch_bounds__(256) void sign_normalise_kernel(const float* __restrict__ Afac, long lda, int n,
                                                             float* __restrict__ R, long ldr, float* __restrict__ U,
                                                             long ldu, unsigned* flags) {
    const long total = (long)n * n;
    for (long e = (long)blockIdx.x * 256 + threadIdx.x; e < total; e += (long)gridDim.x * 256) {
        const int r = (int)(e / n), c = (int)(e % n);
        const float dc = Afac[(long)c * lda + c];
        const float sc = dc >= 0.f ? 1.f : -1.f;
        R[(long)r * ldr + c] *= sc;
        if (U != nullptr) {
            const float dr = Afac[(long)r * lda + r];
            const float sr = dr >= 0.f ? 1.f : -1.f;
            U[(long)r * ldu + c] = (c >= r) ? sr * Afac[(long)r * lda + c] : 0.f;
        }
        if (r == c) {
            if (!(fabsf(dc) <= 3.0e38f)) atomicOr(flags, DQ_FLAG_NONFINITE);
            else if (dc == 0.f) atomicOr(flags, DQ_FLAG_SINGULAR);
        }
    }
}

inline unsigned grid_for(long total) {
    long b = (total + 255) / 256;
    if (b > 8192) b = 8192;
    if (b < 1) b = 1;
    return (unsigned)b;
}

}  // namespace

size_t panel_scratch_floats(int /*m*/) { return (size_t)kPanel * (8192 + 64); }

template <int NT, int Q, int SW, int VCH = Q>
static void launch_panel_cfg(float* A, long lda, int m, int jb, float* tau, float* vscratch, float* tslices,
                             unsigned* flags, int vec, hipStream_t s) {
    hipLaunchKernelGGL((qr_panel_kernel<NT, Q, SW, VCH>), dim3(1), dim3(NT), 0, s, A, lda, m, jb, tau, vscratch, tslices,
                       flags, vec);
}

static hipError_t finish_panel(float* A, long lda, int m, int jb, const float* vscratch, int mp, int sw, int vec,
                               hipStream_t s) {
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || m <= jb) return e;
    const long total = (long)(m - jb) * ((jb + 3) / 4);
    long blocks = (total + 255) / 256;
    if (blocks > 2048) blocks = 2048;
    hipLaunchKernelGGL(unpack_reflectors_kernel, dim3((unsigned)blocks), dim3(256), 0, s, A, lda, m, jb, vscratch, mp, sw, vec);
    return hipGetLastError();
}

hipError_t launch_qr_panel(float* A, long lda, int m, int jb, float* tau, float* vscratch, float* tslices,
                           int* slice_width, unsigned* flags, hipStream_t s) {
    if (m <= 0 || jb <= 0) return hipSuccess;
    if (m > 8192 || jb > kPanel || jb > m) return hipErrorInvalidValue;
    const int vec = ((reinterpret_cast<uintptr_t>(A) & 15) == 0 && (lda & 3) == 0) ? 1 : 0;
    constexpr int NT = 512;
    int mp, sw = 8;
    // rows per thread Q = 1, 2, 4, 8 with 8-column slices; taller panels (m > 4096) use Q = 16 with 4-column slices,
    // which is what fits the register file (an 8-column slice of 16 rows per thread plus the 64 projection sums spill)
    if (m <= NT * 1) { launch_panel_cfg<NT, 1, 8>(A, lda, m, jb, tau, vscratch, tslices, flags, vec, s); mp = NT * 1; }
    else if (m <= NT * 2) { launch_panel_cfg<NT, 2, 8>(A, lda, m, jb, tau, vscratch, tslices, flags, vec, s); mp = NT * 2; }
    else if (m <= NT * 4) { launch_panel_cfg<NT, 4, 8>(A, lda, m, jb, tau, vscratch, tslices, flags, vec, s); mp = NT * 4; }
    else if (m <= NT * 8) { launch_panel_cfg<NT, 8, 8>(A, lda, m, jb, tau, vscratch, tslices, flags, vec, s); mp = NT * 8; }
    else { launch_panel_cfg<NT, 16, 4>(A, lda, m, jb, tau, vscratch, tslices, flags, vec, s); mp = NT * 16; sw = 4; }
    *slice_width = sw;
    return finish_panel(A, lda, m, jb, vscratch, mp, sw, vec, s);
}

hipError_t launch_tfactor(const float* gpart, int splits, long stride, long ldp, int jb, int nla,
                          const float* tslices, int slice_width, float* Tout, float* W2out, hipStream_t s) {
    hipLaunchKernelGGL(tfactor_kernel, dim3(1), dim3(1024), 0, s, gpart, splits, stride, ldp, jb, nla, tslices,
                       slice_width, Tout, W2out);
    return hipGetLastError();
}

hipError_t launch_copy2d(const float* src, long lds, float* dst, long ldd, int rows, int cols, hipStream_t s) {
    if (rows <= 0 || cols <= 0) return hipSuccess;
    const long total4 = (long)rows * (cols / 4);
    if (cols % 4 == 0 && (ldd & 3) == 0 && (reinterpret_cast<uintptr_t>(dst) & 15) == 0 && total4 < (1L << 31) &&
        (src == nullptr || ((lds & 3) == 0 && (reinterpret_cast<uintptr_t>(src) & 15) == 0))) {
        hipLaunchKernelGGL(copy2d_vec_kernel, dim3(grid_for(total4)), dim3(256), 0, s, src, lds, dst, ldd, (unsigned)total4,
                           (unsigned)(cols / 4));
        return hipGetLastError();
    }
    hipLaunchKernelGGL(copy2d_kernel, dim3(grid_for((long)rows * cols)), dim3(256), 0, s, src, lds, dst, ldd, rows, cols);
    return hipGetLastError();
}

hipError_t launch_set_identity(float* A, long lda, int n, hipStream_t s) {
    const long total4 = (long)n * (n / 4);
    if (n % 4 == 0 && (lda & 3) == 0 && (reinterpret_cast<uintptr_t>(A) & 15) == 0 && total4 < (1L << 31)) {
        hipLaunchKernelGGL(identity_vec_kernel, dim3(grid_for(total4)), dim3(256), 0, s, A, lda, (unsigned)total4,
                           (unsigned)(n / 4));
        return hipGetLastError();
    }
    hipLaunchKernelGGL(identity_kernel, dim3(grid_for((long)n * n)), dim3(256), 0, s, A, lda, n);
    return hipGetLastError();
}

hipError_t launch_fill_u32(unsigned* p, long count, unsigned v, hipStream_t s) {
    if (count <= 0) return hipSuccess;
    hipLaunchKernelGGL(fill_u32_kernel, dim3(grid_for(count)), dim3(256), 0, s, p, count, v);
    return hipGetLastError();
}

hipError_t launch_sign_normalise(const float* Afac, long lda, int n, float* R, long ldr, float* U, long ldu,
                                 unsigned* flags, hipStream_t s) {
    auto a16 = [](const void* q) { return (reinterpret_cast<uintptr_t>(q) & 15) == 0; };
    if (n % 4 == 0 && lda % 4 == 0 && ldr % 4 == 0 && (U == nullptr || ldu % 4 == 0) && a16(Afac) && a16(R) && a16(U)) {
        const dim3 grid((n + 1023) / 1024, (n + kSignRows - 1) / kSignRows);
        hipLaunchKernelGGL(sign_normalise_vec_kernel, grid, dim3(256), 0, s, Afac, lda, n, R, ldr, U, ldu, flags);
        return hipGetLastError();
    }
    hipLaunchKernelGGL(sign_normalise_kernel, dim3(grid_for((long)n * n)), dim3(256), 0, s, Afac, lda, n, R, ldr, U,
                       ldu, flags);
    return hipGetLastError();
}

}  // namespace dq
