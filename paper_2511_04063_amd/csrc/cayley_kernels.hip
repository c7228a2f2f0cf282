// Elementwise pieces of Cayley SGD with momentum (Alg. 3, App. B.2), the optimiser the paper compares QR-Orth with
// (Sec. 5, optimiser comparison).  Its six n x n products run on the fp32 matrix-core GEMM; what is left are
// HBM-bound passes over n x n matrices: the momentum update, the skew-symmetrisation with the Frobenius norm that the
// step-size rule needs, the step size itself (a device scalar: no host round trip), and sums of two matrices.
#include <math.h>

#include "dq_internal.h"

namespace dq {
namespace {

// M <- beta M - G  (Alg. 3, momentum update)
__global__ __launch_bounds__(256) void cayley_momentum_kernel(float* __restrict__ M, long ldm, const float* __restrict__ G,
                                                             long ldg, int n, float beta) {
    const int q = (n + 3) >> 2;
    const long total = (long)n * q;
    for (long e = (long)blockIdx.x * 256 + threadIdx.x; e < total; e += (long)gridDim.x * 256) {
        const int r = (int)(e / q), c0 = (int)(e % q) << 2;
#pragma unroll
        for (int j = 0; j < 4; ++j)
            if (c0 + j < n) M[(long)r * ldm + c0 + j] = beta * M[(long)r * ldm + c0 + j] - G[(long)r * ldg + c0 + j];
    }
}

// W = What - What^T (Alg. 3, skew-symmetrisation) on 32 x 32 tiles: tile (bi, bj) and its mirror are both read row-wise (coalesced)
// and the mirror is transposed through LDS.  Each block also leaves the sum of squares of the entries it wrote.
__global__ __launch_bounds__(256) void cayley_skew_kernel(const float* __restrict__ H, long ldh, int n, float* __restrict__ W,
                                                         long ldw, double* __restrict__ partials) {
    __shared__ float mirror[32][33];
    __shared__ float wsum[4];
    const int tiles = (n + 31) >> 5;
    const int bi = blockIdx.x / tiles, bj = blockIdx.x % tiles;
    const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;
    for (int i = ty; i < 32; i += 8) {
        const int r = bj * 32 + i, c = bi * 32 + tx;        // the mirror tile (bj, bi)
        mirror[i][tx] = (r < n && c < n) ? H[(long)r * ldh + c] : 0.f;
    }
    __syncthreads();
    float acc = 0.f;
    for (int i = ty; i < 32; i += 8) {
        const int r = bi * 32 + i, c = bj * 32 + tx;
        if (r < n && c < n) {
            const float w = H[(long)r * ldh + c] - mirror[tx][i];
            W[(long)r * ldw + c] = w;
            acc += w * w;
        }
    }
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) acc += __shfl_xor(acc, o);
    if ((threadIdx.x & 63) == 0) wsum[threadIdx.x >> 6] = acc;
    __syncthreads();
    if (threadIdx.x == 0) partials[blockIdx.x] = ((double)wsum[0] + (double)wsum[1]) + ((double)wsum[2] + (double)wsum[3]);
}

// alpha = min(lr, 2 q / (||W||_F + eps))  (Alg. 3, step-size rule); out[0] = alpha, out[1] = alpha / 2
__global__ __launch_bounds__(256) void cayley_alpha_kernel(const double* __restrict__ partials, int count, float lr, float q,
                                                          float eps, float* __restrict__ out) {
    __shared__ double sh[256];
    double t = 0.0;
    for (int i = threadIdx.x; i < count; i += 256) t += partials[i];
    sh[threadIdx.x] = t;
    __syncthreads();
    for (int o = 128; o >= 1; o >>= 1) {
        if ((int)threadIdx.x < o) sh[threadIdx.x] += sh[threadIdx.x + o];
        __syncthreads();
    }
    if (threadIdx.x == 0) {
        const float norm = (float)sqrt(sh[0]);
        const float cap = 2.f * q / (norm + eps);
        const float alpha = lr < cap ? lr : cap;        // a NaN norm leaves lr
        out[0] = alpha;
        out[1] = 0.5f * alpha;
    }
}

// out = A + scale B
__global__ __launch_bounds__(256) void add_scaled_kernel(float* out, long ldo, const float* A, long lda, const float* B,
                                                        long ldb, int n, float scale_host, const float* __restrict__ scale_dev) {
    const float sc = scale_dev != nullptr ? scale_host * *scale_dev : scale_host;
    const int q = (n + 3) >> 2;
    const long total = (long)n * q;
    for (long e = (long)blockIdx.x * 256 + threadIdx.x; e < total; e += (long)gridDim.x * 256) {
        const int r = (int)(e / q), c0 = (int)(e % q) << 2;
#pragma unroll
        for (int j = 0; j < 4; ++j)
            if (c0 + j < n) out[(long)r * ldo + c0 + j] = A[(long)r * lda + c0 + j] + sc * B[(long)r * ldb + c0 + j];
    }
}

unsigned elementwise_grid(int n) {
    long b = ((long)n * ((n + 3) / 4) + 255) / 256;
    if (b > 8192) b = 8192;
    return (unsigned)(b < 1 ? 1 : b);
}

}  // namespace

hipError_t launch_cayley_momentum(float* M, long ldm, const float* G, long ldg, int n, float beta, hipStream_t s) {
    hipLaunchKernelGGL(cayley_momentum_kernel, dim3(elementwise_grid(n)), dim3(256), 0, s, M, ldm, G, ldg, n, beta);
    return hipGetLastError();
}

int cayley_skew_grid(int n) {
    const int tiles = (n + 31) / 32;
    return tiles * tiles;
}

hipError_t launch_cayley_skew(const float* What, long ldh, int n, float* W, long ldw, double* partials, hipStream_t s) {
    hipLaunchKernelGGL(cayley_skew_kernel, dim3(cayley_skew_grid(n)), dim3(256), 0, s, What, ldh, n, W, ldw, partials);
    return hipGetLastError();
}

hipError_t launch_cayley_alpha(const double* partials, int count, float lr, float q, float eps, float* alpha_dev,
                               hipStream_t s) {
    hipLaunchKernelGGL(cayley_alpha_kernel, dim3(1), dim3(256), 0, s, partials, count, lr, q, eps, alpha_dev);
    return hipGetLastError();
}

hipError_t launch_add_scaled(float* out, long ldo, const float* A, long lda, const float* B, long ldb, int n,
                             float scale_host, const float* scale_dev, hipStream_t s) {
    hipLaunchKernelGGL(add_scaled_kernel, dim3(elementwise_grid(n)), dim3(256), 0, s, out, ldo, A, lda, B, ldb, n,
                       scale_host, scale_dev);
    return hipGetLastError();
}

}  // namespace dq
