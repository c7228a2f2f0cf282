// HBM-bound passes of the step:
//   * the fused Whip loss + gradient pass over Y (Eq. 4 and its derivative; the loss step of Alg. 1),
//   * the two-plane bf16 split of the rotation with a transpose (operand preparation for X @ R),
//   * P = strict_lower(B - B^T) of the derivative through Z = R U,
//   * inverses of the diagonal blocks of U for the blocked triangular solve,
//   * the SGD update Z <- Z - eta dZ (the last step of Alg. 1).
#include <math.h>
#include <stdlib.h>

#include "dq_internal.h"
#include "dq_small64.h"

namespace dq {
namespace {

__device__ __forceinline__ uint32_t f32_to_bf16_rne(float f) {
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (u >> 16) | 0x40u;   // NaN stays NaN
    u += 0x7fffu + ((u >> 16) & 1u);
    return u >> 16;
}

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) v += __shfl_xor(v, o);
    return v;
}

// Each thread handles runs of 8 consecutive elements of a row: two 16-byte loads of Y, one 16-byte (bf16)
// or two 16-byte (fp32) stores of dY.  e = exp(-|y|) contributes to the loss; dY = -scale * sgn(y) * e.
template <bool BF16OUT>
__global__ __launch_bounds__(256) void whip_kernel(const float* __restrict__ Y, long ldy, int T, int n, float scale,
                                                   void* __restrict__ dYv, long lddy, double* __restrict__ partials,
                                                   int yvec, int dvec, long sy, long sdy) {
    // blockIdx.y: problem of a batch (element strides sy, sdy; gridDim.x partials per problem)
    Y += (long)blockIdx.y * sy;
    dYv = static_cast<char*>(dYv) + (long)blockIdx.y * sdy * (BF16OUT ? 2 : 4);
    partials += (long)blockIdx.y * gridDim.x;
    const int cpr = (n + 7) >> 3;                 // 8-element chunks per row
    const long chunks = (long)T * cpr;
    float acc = 0.f;
    if (BF16OUT && yvec > 1 && dvec && (n & 7) == 0 && ldy == n && lddy == n) {
        // Dense rows: one flat stream, no row/column arithmetic.  Consecutive lanes take consecutive 16-byte pieces
        // (every load instruction covers 1 KiB without gaps), four pieces per thread in flight, and the hardware's
        // packed round-to-nearest-even conversion packs 4 results into an 8-byte store.
        typedef float f32x2 __attribute__((ext_vector_type(2)));
        typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
        const float4* src = reinterpret_cast<const float4*>(Y);
        uint2* dst = reinterpret_cast<uint2*>(dYv);
        const long total4 = (long)T * (n >> 2);
        constexpr int U = 8;
        const long stride = 256;    // a workgroup takes U consecutive 4 KiB pieces per iteration
        for (long p0 = (long)blockIdx.x * (256 * U) + threadIdx.x; p0 < total4; p0 += (long)gridDim.x * (256 * U)) {
            float4 q[U];
#pragma unroll
            for (int h = 0; h < U; ++h)
            {
                if (p0 + h * stride >= total4) {
                    q[h] = make_float4(0.f, 0.f, 0.f, 0.f);
                } else if (yvec > 2) {
                    // a Y larger than the last-level cache is streamed: nontemporal loads leave the cache to the
                    // writes of dY (805 MB case: 150 -> 126 us; slower by 10 % when Y is cache-resident)
                    typedef float f32x4 __attribute__((ext_vector_type(4)));
                    const f32x4 v = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(Y) + p0 + h * stride);
                    q[h] = make_float4(v.x, v.y, v.z, v.w);
                } else {
                    q[h] = src[p0 + h * stride];
                }
            }
#pragma unroll
            for (int h = 0; h < U; ++h) {
                const bool live = p0 + h * stride < total4;
                const float yv[4] = {q[h].x, q[h].y, q[h].z, q[h].w};
                float dv[4];
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const float ex = __expf(-fabsf(yv[j]));
                    if (live) acc += ex;
                    const float sg = (yv[j] > 0.f) ? -scale : ((yv[j] < 0.f) ? scale : 0.f);
                    dv[j] = sg * ex;
                }
                f32x2 a0 = {dv[0], dv[1]}, a1 = {dv[2], dv[3]};
                const bf16x2 b0 = __builtin_convertvector(a0, bf16x2), b1 = __builtin_convertvector(a1, bf16x2);
                if (live)
                    dst[p0 + h * stride] = make_uint2(*reinterpret_cast<const uint32_t*>(&b0),
                                                      *reinterpret_cast<const uint32_t*>(&b1));
            }
        }
    } else
    for (long e = (long)blockIdx.x * 256 + threadIdx.x; e < chunks; e += (long)gridDim.x * 256) {
        const int row = (int)(e / cpr);
        const int c0 = (int)(e - (long)row * cpr) << 3;
        const float* src = Y + (long)row * ldy + c0;
        float y[8];
        const bool full = c0 + 7 < n;
        if (full && yvec) {
            const float4 a = *reinterpret_cast<const float4*>(src);
            const float4 b = *reinterpret_cast<const float4*>(src + 4);
            y[0] = a.x; y[1] = a.y; y[2] = a.z; y[3] = a.w; y[4] = b.x; y[5] = b.y; y[6] = b.z; y[7] = b.w;
        } else {
#pragma unroll
            for (int j = 0; j < 8; ++j) y[j] = (c0 + j < n) ? src[j] : 0.f;
        }
        float d[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const float ay = fabsf(y[j]);
            const float ex = __expf(-ay);
            if (c0 + j < n) acc += ex;
            const float sg = (y[j] > 0.f) ? -scale : ((y[j] < 0.f) ? scale : 0.f);
            d[j] = sg * ex;
        }
        if (BF16OUT) {
            bf16_t* dst = reinterpret_cast<bf16_t*>(dYv) + (long)row * lddy + c0;
            if (full && dvec) {
                uint4 o;
                o.x = f32_to_bf16_rne(d[0]) | (f32_to_bf16_rne(d[1]) << 16);
                o.y = f32_to_bf16_rne(d[2]) | (f32_to_bf16_rne(d[3]) << 16);
                o.z = f32_to_bf16_rne(d[4]) | (f32_to_bf16_rne(d[5]) << 16);
                o.w = f32_to_bf16_rne(d[6]) | (f32_to_bf16_rne(d[7]) << 16);
                *reinterpret_cast<uint4*>(dst) = o;
            } else {
#pragma unroll
                for (int j = 0; j < 8; ++j)
                    if (c0 + j < n) dst[j] = (bf16_t)f32_to_bf16_rne(d[j]);
            }
        } else {
            float* dst = reinterpret_cast<float*>(dYv) + (long)row * lddy + c0;
            if (full && dvec) {
                *reinterpret_cast<float4*>(dst) = make_float4(d[0], d[1], d[2], d[3]);
                *reinterpret_cast<float4*>(dst + 4) = make_float4(d[4], d[5], d[6], d[7]);
            } else {
#pragma unroll
                for (int j = 0; j < 8; ++j)
                    if (c0 + j < n) dst[j] = d[j];
            }
        }
    }
    __shared__ float wsum[4];
    acc = wave_sum(acc);
    if ((threadIdx.x & 63) == 0) wsum[threadIdx.x >> 6] = acc;
    __syncthreads();
    if (threadIdx.x == 0) partials[blockIdx.x] = (double)wsum[0] + (double)wsum[1] + (double)wsum[2] + (double)wsum[3];
}

__global__ __launch_bounds__(256) void loss_finish_kernel(const double* __restrict__ partials, int count, float scale,
                                                          float* __restrict__ loss_dev, unsigned* flags) {
    __shared__ double sh[256];
    partials += (long)blockIdx.x * count;   // one workgroup per problem of a batch
    loss_dev += blockIdx.x;
    double t = 0.0;
    for (int i = threadIdx.x; i < count; i += 256) t += partials[i];
    sh[threadIdx.x] = t;
    __syncthreads();
    for (int o = 128; o >= 1; o >>= 1) {
        if ((int)threadIdx.x < o) sh[threadIdx.x] += sh[threadIdx.x + o];
        __syncthreads();
    }
    if (threadIdx.x == 0) {
        const double L = (double)scale * sh[0];
        const float Lf = (float)L;
        *loss_dev = Lf;
        if (!(fabsf(Lf) <= 3.0e38f)) atomicOr(flags, DQ_FLAG_NONFINITE);
    }
}

// Two-plane bf16 split of R, transposed, through a 32 x 33 LDS tile so that both the read and the writes are
// coalesced:  RbT[j][k] = hi(R[k][j]),  RbT[j][koff + k] = lo(R[k][j]);  hi + lo carries 16 mantissa bits of R.
// The grid covers k up to koff, so the padding columns [n, koff) of both planes are written as zero.
__global__ __launch_bounds__(256) void split_transpose_bf16_kernel(const float* __restrict__ R, long ldr, int n,
                                                                   bf16_t* __restrict__ RbT, long ldt, int koff) {
    __shared__ float tile[32][33];
    const int bx = blockIdx.x * 32, by = blockIdx.y * 32;   // bx: column block of R (j), by: row block of R (k)
    const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;
    for (int i = ty; i < 32; i += 8) {
        const int r = by + i, c = bx + tx;
        tile[i][tx] = (r < n && c < n) ? R[(long)r * ldr + c] : 0.f;
    }
    __syncthreads();
    for (int i = ty; i < 32; i += 8) {
        const int j = bx + i, k = by + tx;
        if (j < n && k < koff) {
            const float r = tile[tx][i];
            const uint32_t hi = f32_to_bf16_rne(r);
            const float rem = r - __uint_as_float(hi << 16);
            RbT[(long)j * ldt + k] = (bf16_t)hi;
            RbT[(long)j * ldt + koff + k] = (bf16_t)f32_to_bf16_rne(rem);
        }
    }
}

// The same for n a multiple of 64, koff == n and 16-byte aligned rows on both sides: 64 x 64 tiles, 16-byte loads, and
// every thread writes eight consecutive entries of an output row per plane.
__global__ __launch_bounds__(256) void split_transpose64_bf16_kernel(const float* __restrict__ R, long ldr,
                                                                     bf16_t* __restrict__ RbT, long ldt, int koff) {
    __shared__ float tile[64][65];
    const int bx = blockIdx.x * 64, by = blockIdx.y * 64;   // bx: column block of R (j), by: row block of R (k)
    const int tid = threadIdx.x;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int f = tid + 256 * i;
        const int r = f >> 4, c = (f & 15) << 2;
        const float4 v = *reinterpret_cast<const float4*>(R + (long)(by + r) * ldr + bx + c);
        tile[r][c] = v.x; tile[r][c + 1] = v.y; tile[r][c + 2] = v.z; tile[r][c + 3] = v.w;
    }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int f = tid + 256 * i;
        const int j = f >> 3, k0 = (f & 7) << 3;
        uint32_t wh[4], wl[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const float r0 = tile[k0 + 2 * q][j], r1 = tile[k0 + 2 * q + 1][j];
            const uint32_t h0 = f32_to_bf16_rne(r0), h1 = f32_to_bf16_rne(r1);
            const uint32_t l0 = f32_to_bf16_rne(r0 - __uint_as_float(h0 << 16));
            const uint32_t l1 = f32_to_bf16_rne(r1 - __uint_as_float(h1 << 16));
            wh[q] = h0 | (h1 << 16); wl[q] = l0 | (l1 << 16);
        }
        bf16_t* o = RbT + (long)(bx + j) * ldt + by + k0;
        *reinterpret_cast<uint4*>(o) = make_uint4(wh[0], wh[1], wh[2], wh[3]);
        *reinterpret_cast<uint4*>(o + koff) = make_uint4(wl[0], wl[1], wl[2], wl[3]);
    }
}

// Three-plane bf16 split of an fp32 matrix (a = a1 + a2 + a3 to 24 mantissa bits; both subtractions are exact in fp32).
__device__ __forceinline__ void split3(float a, bf16_t& p1, bf16_t& p2, bf16_t& p3) {
    const uint32_t h1 = f32_to_bf16_rne(a);
    const float r1 = a - __uint_as_float(h1 << 16);
    const uint32_t h2 = f32_to_bf16_rne(r1);
    const float r2 = r1 - __uint_as_float(h2 << 16);
    p1 = (bf16_t)h1; p2 = (bf16_t)h2; p3 = (bf16_t)f32_to_bf16_rne(r2);
}

// planes of A^T through a 32 x 33 LDS tile (coalesced on both sides); any shape
__global__ __launch_bounds__(256) void split3_transpose_bf16_kernel(const float* __restrict__ A, long lda, int rows, int cols,
                                                                    bf16_t* __restrict__ out, long ldo, long plane) {
    __shared__ float tile[32][33];
    const int bx = blockIdx.x * 32, by = blockIdx.y * 32;   // bx: column block of A, by: row block of A
    const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;
    for (int i = ty; i < 32; i += 8) {
        const int r = by + i, c = bx + tx;
        tile[i][tx] = (r < rows && c < cols) ? A[(long)r * lda + c] : 0.f;
    }
    __syncthreads();
    for (int i = ty; i < 32; i += 8) {
        const int j = bx + i, k = by + tx;
        if (j < cols && k < rows) {
            bf16_t p1, p2, p3;
            split3(tile[tx][i], p1, p2, p3);
            bf16_t* o = out + (long)j * ldo + k;
            o[0] = p1; o[plane] = p2; o[2 * plane] = p3;
        }
    }
}

// The same for rows and cols multiples of 64 with 16-byte aligned rows on both sides: 64 x 64 tiles, 16-byte loads, and
// every thread writes eight consecutive entries of an output row per plane (16 bytes; the eight threads of a row 128).
__global__ __launch_bounds__(256) void split3_transpose64_bf16_kernel(const float* __restrict__ A, long lda,
                                                                      bf16_t* __restrict__ out, long ldo, long plane) {
    __shared__ float tile[64][65];
    const int bx = blockIdx.x * 64, by = blockIdx.y * 64;   // bx: column block of A, by: row block of A
    const int tid = threadIdx.x;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int f = tid + 256 * i;
        const int r = f >> 4, c = (f & 15) << 2;
        const float4 v = *reinterpret_cast<const float4*>(A + (long)(by + r) * lda + bx + c);
        tile[r][c] = v.x; tile[r][c + 1] = v.y; tile[r][c + 2] = v.z; tile[r][c + 3] = v.w;
    }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int f = tid + 256 * i;
        const int j = f >> 3, k0 = (f & 7) << 3;            // output row bx + j, entries by + k0 .. + 7
        uint32_t w1[4], w2[4], w3[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            bf16_t a1, a2, a3, b1, b2, b3;
            split3(tile[k0 + 2 * q][j], a1, a2, a3);
            split3(tile[k0 + 2 * q + 1][j], b1, b2, b3);
            w1[q] = a1 | ((uint32_t)b1 << 16); w2[q] = a2 | ((uint32_t)b2 << 16); w3[q] = a3 | ((uint32_t)b3 << 16);
        }
        bf16_t* o = out + (long)(bx + j) * ldo + by + k0;
        *reinterpret_cast<uint4*>(o) = make_uint4(w1[0], w1[1], w1[2], w1[3]);
        *reinterpret_cast<uint4*>(o + plane) = make_uint4(w2[0], w2[1], w2[2], w2[3]);
        *reinterpret_cast<uint4*>(o + 2 * plane) = make_uint4(w3[0], w3[1], w3[2], w3[3]);
    }
}

// planes of A itself, four entries per thread (cols a multiple of 4, 16-byte aligned rows of A, 8-byte of out)
__global__ __launch_bounds__(256) void split3_bf16_kernel(const float* __restrict__ A, long lda, int rows, int cols4,
                                                          bf16_t* __restrict__ out, long ldo, long plane) {
    const long total = (long)rows * cols4;
    for (long e = (long)blockIdx.x * 256 + threadIdx.x; e < total; e += (long)gridDim.x * 256) {
        const int r = (int)(e / cols4), c = (int)(e % cols4) * 4;
        const float4 v = *reinterpret_cast<const float4*>(A + (long)r * lda + c);
        bf16_t a[4], b[4], d[4];
        split3(v.x, a[0], b[0], d[0]); split3(v.y, a[1], b[1], d[1]);
        split3(v.z, a[2], b[2], d[2]); split3(v.w, a[3], b[3], d[3]);
        bf16_t* o = out + (long)r * ldo + c;
        *reinterpret_cast<uint2*>(o) = make_uint2(a[0] | ((uint32_t)a[1] << 16), a[2] | ((uint32_t)a[3] << 16));
        *reinterpret_cast<uint2*>(o + plane) = make_uint2(b[0] | ((uint32_t)b[1] << 16), b[2] | ((uint32_t)b[3] << 16));
        *reinterpret_cast<uint2*>(o + 2 * plane) = make_uint2(d[0] | ((uint32_t)d[1] << 16), d[2] | ((uint32_t)d[3] << 16));
    }
}

// dst (cols x rows) = src^T for a rows x cols bf16 matrix, 64 x 64 tiles through LDS with 16-byte loads and stores.
// rows and cols are multiples of 64, both leading dimensions multiples of 8 and both pointers 16-byte aligned.
// Operand preparation for G = X^T dY (the loss step of Alg. 1): with both operands stored token-contiguous the product reads
// rows only.
__global__ __launch_bounds__(256) void transpose_bf16_kernel(const bf16_t* __restrict__ src, long lds_, int rows,
                                                             int cols, bf16_t* __restrict__ dst, long ldd) {
    constexpr int S = 66;   // row stride of the tile in elements: 33 words, odd
    __shared__ __align__(16) unsigned short tile[64 * S];
    const int tiles_c = cols >> 6;
    const int r0 = (blockIdx.x / tiles_c) << 6, c0 = (blockIdx.x % tiles_c) << 6;
    const int tid = threadIdx.x;
    const int part = tid & 7, line = tid >> 3;
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        const int r = line + 32 * h;
        const uint4 v = *reinterpret_cast<const uint4*>(src + (long)(r0 + r) * lds_ + c0 + part * 8);
        uint32_t* t = reinterpret_cast<uint32_t*>(tile + r * S + part * 8);
        t[0] = v.x; t[1] = v.y; t[2] = v.z; t[3] = v.w;
    }
    __syncthreads();
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        const int c = line + 32 * h;   // column of src = row of dst
        uint32_t w[4];
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const uint32_t lo = tile[(part * 8 + 2 * k) * S + c];
            const uint32_t hi = tile[(part * 8 + 2 * k + 1) * S + c];
            w[k] = lo | (hi << 16);
        }
        *reinterpret_cast<uint4*>(dst + (long)(c0 + c) * ldd + r0 + part * 8) = make_uint4(w[0], w[1], w[2], w[3]);
    }
}

// Z[i][j] = s[i] * (-1)^popcount(i & j) * c  with c = 1 / sqrt(n): a randomised Hadamard matrix (Sylvester construction,
// n a power of two), the initial latent of the paper's runs (App., hyper-parameter settings).  The signs are an input.
__global__ __launch_bounds__(256) void hadamard_init_kernel(const float* __restrict__ sgn, int n, float c,
                                                            float* __restrict__ Z, long ldz) {
    const long total = (long)n * n;
    for (long e = (long)blockIdx.x * 256 + threadIdx.x; e < total; e += (long)gridDim.x * 256) {
        const int i = (int)(e / n), j = (int)(e % n);
        const float h = (__popc((unsigned)(i & j)) & 1) ? -c : c;
        Z[(long)i * ldz + j] = sgn[i] * h;
    }
}

// count += #{(t, c) : |Y[t][c]| > tau}: the objective the calibration is a smooth stand-in for (Sec. 4.1, Eq. 1), used
// as an evaluation metric.  Integer atomics: the result does not depend on the order of the additions.
__global__ __launch_bounds__(256) void outlier_count_kernel(const float* __restrict__ Y, long ldy, int T, int n, float tau,
                                                            unsigned long long* __restrict__ count) {
    const int cpr = (n + 3) >> 2;
    const long chunks = (long)T * cpr;
    const bool vec = (reinterpret_cast<uintptr_t>(Y) & 15) == 0 && (ldy & 3) == 0;
    unsigned local = 0;
    for (long e = (long)blockIdx.x * 256 + threadIdx.x; e < chunks; e += (long)gridDim.x * 256) {
        const int row = (int)(e / cpr);
        const int c0 = (int)(e - (long)row * cpr) << 2;
        const float* src = Y + (long)row * ldy + c0;
        if (vec && c0 + 3 < n) {
            const float4 v = *reinterpret_cast<const float4*>(src);
            local += (fabsf(v.x) > tau) + (fabsf(v.y) > tau) + (fabsf(v.z) > tau) + (fabsf(v.w) > tau);
        } else {
            for (int j = 0; j < 4; ++j)
                if (c0 + j < n) local += fabsf(src[j]) > tau;
        }
    }
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) local += __shfl_xor(local, o);
    if ((threadIdx.x & 63) == 0 && local != 0) atomicAdd(count, (unsigned long long)local);
}

// out[t][:] = src[idx[t]][:] for t < rows_out: the token-sampling step in front of the loop (Alg. 1) as a
// gather of whole rows, 16 bytes per lane (row_bytes is a multiple of 16, rows 16-byte aligned).  An index outside
// [0, rows_in) copies nothing for that row and raises the flag.
__global__ __launch_bounds__(256) void gather_rows_kernel(const char* __restrict__ src, long src_stride, int rows_in,
                                                          const int* __restrict__ idx, int rows_out, int row_bytes,
                                                          char* __restrict__ out, long out_stride, int rows_per_block,
                                                          unsigned* flags) {
    const int pieces = row_bytes >> 4;
    const int tpr = 256 / rows_per_block;             // threads per row
    const int rsub = threadIdx.x / tpr, lane = threadIdx.x % tpr;
    if (rsub >= rows_per_block) return;
    for (long t = (long)blockIdx.x * rows_per_block + rsub; t < rows_out; t += (long)gridDim.x * rows_per_block) {
        const int r = idx[t];
        if (r < 0 || r >= rows_in) {
            if (lane == 0) atomicOr(flags, DQ_FLAG_BAD_INDEX);
            continue;
        }
        const uint4* s4 = reinterpret_cast<const uint4*>(src + (long)r * src_stride);
        uint4* d4 = reinterpret_cast<uint4*>(out + t * out_stride);
        for (int p = lane; p < pieces; p += tpr) d4[p] = s4[p];
    }
}

// P[i][j] = B[i][j] - B[j][i] for i > j, else 0.  Mzero (optional) is cleared.  blockIdx.z: problem of a batch.
__global__ __launch_bounds__(256) void skew_lower_kernel(const float* __restrict__ B, long ldb, int n,
                                                         float* __restrict__ P, long ldp, float* __restrict__ Mz,
                                                         long ldm, long sb, long sp, long sm) {
    __shared__ float tile[32][33];
    B += (long)blockIdx.z * sb;
    P += (long)blockIdx.z * sp;
    if (Mz != nullptr) Mz += (long)blockIdx.z * sm;
    const int bx = blockIdx.x * 32, by = blockIdx.y * 32;   // output tile: rows by.., cols bx..
    const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;
    const bool need = by + 31 > bx;   // some i > j in this tile
    if (need) {
        // transposed source tile: B[bx + i][by + tx]
        for (int i = ty; i < 32; i += 8) {
            const int r = bx + i, c = by + tx;
            tile[i][tx] = (r < n && c < n) ? B[(long)r * ldb + c] : 0.f;
        }
    }
    __syncthreads();
    for (int i = ty; i < 32; i += 8) {
        const int r = by + i, c = bx + tx;
        if (r < n && c < n) {
            float v = 0.f;
            if (need && r > c) v = B[(long)r * ldb + c] - tile[tx][i];
            P[(long)r * ldp + c] = v;
            if (Mz != nullptr) Mz[(long)r * ldm + c] = 0.f;
        }
    }
}

// The same for n a multiple of 64 and 16-byte aligned rows everywhere: 64 x 64 tiles, 16-byte loads and stores.
__global__ __launch_bounds__(256) void skew_lower64_kernel(const float* __restrict__ B, long ldb, float* __restrict__ P,
                                                           long ldp, float* __restrict__ Mz, long ldm, long sb, long sp,
                                                           long sm) {
    __shared__ float tile[64][65];
    B += (long)blockIdx.z * sb;
    P += (long)blockIdx.z * sp;
    if (Mz != nullptr) Mz += (long)blockIdx.z * sm;
    const int bx = blockIdx.x * 64, by = blockIdx.y * 64;   // output tile: rows by.., cols bx..
    const int tid = threadIdx.x;
    const bool need = by + 63 > bx;                          // some i > j in this tile
    if (need) {
#pragma unroll
        for (int q = 0; q < 4; ++q) {                        // the transposed source tile: B[bx + r][by + c .. c + 3]
            const int f = tid + 256 * q, r = f >> 4, c = (f & 15) << 2;
            const float4 v = *reinterpret_cast<const float4*>(B + (long)(bx + r) * ldb + by + c);
            tile[r][c] = v.x; tile[r][c + 1] = v.y; tile[r][c + 2] = v.z; tile[r][c + 3] = v.w;
        }
    }
    __syncthreads();
    const float4 zero = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const int f = tid + 256 * q, r = f >> 4, c = (f & 15) << 2;
        const int gr = by + r, gc = bx + c;
        float4 v = zero;
        if (need && gr > gc) {
            const float4 b = *reinterpret_cast<const float4*>(B + (long)gr * ldb + gc);
            v.x = b.x - tile[c][r];
            if (gr > gc + 1) v.y = b.y - tile[c + 1][r];
            if (gr > gc + 2) v.z = b.z - tile[c + 2][r];
            if (gr > gc + 3) v.w = b.w - tile[c + 3][r];
        }
        *reinterpret_cast<float4*>(P + (long)gr * ldp + gc) = v;
        if (Mz != nullptr) *reinterpret_cast<float4*>(Mz + (long)gr * ldm + gc) = zero;
    }
}

// Inverse of one 128 x 128 diagonal block (w x w used, w <= kTrsmBlock) of an upper-triangular matrix, one
// workgroup per block:  inv [[A, B], [0, C]] = [[A^-1, -A^-1 B C^-1], [0, C^-1]]  with the 64 x 64 inverses and the
// two products done out of LDS on the matrix cores.  Rows and columns beyond w are padded with the identity for
// the computation and written as zero.  A zero pivot raises DQ_FLAG_SINGULAR (the result is then not finite).
static_assert(kTrsmBlock == 2 * B64, "the block inverse is built from 64 x 64 pieces");
__device__ __forceinline__ void load_block64(const float* __restrict__ Ub, long ldu, int w, int r0, int c0, float* dst,
                                             int tid) {
#pragma unroll
    for (int q = 0; q < 16; ++q) {
        const int e = tid + NTHR * q;
        const int i = r0 + (e >> 6), j = c0 + (e & 63);
        dst[(e >> 6) * LS + (e & 63)] = (i < w && j < w) ? Ub[(long)i * ldu + j] : (i == j ? 1.f : 0.f);
    }
    __syncthreads();
}
__device__ __forceinline__ void store_block64(const float* src, float* __restrict__ out, int w, int r0, int c0, int tid) {
#pragma unroll
    for (int q = 0; q < 16; ++q) {
        const int e = tid + NTHR * q;
        const int i = r0 + (e >> 6), j = c0 + (e & 63);
        out[(long)i * kTrsmBlock + j] = (i < w && j < w) ? src[(e >> 6) * LS + (e & 63)] : 0.f;
    }
}
__global__ __launch_bounds__(NTHR) void trinv_blocks_kernel(const float* __restrict__ U, long ldu, int n,
                                                            float* __restrict__ Uinv, unsigned* flags, long su,
                                                            long sinv) {
    U += (long)blockIdx.y * su;       // problem of a batch
    Uinv += (long)blockIdx.y * sinv;
    __shared__ float Bs[3 * B64 * LS];
    float* B0 = Bs;
    float* B1 = Bs + B64 * LS;
    float* B2 = Bs + 2 * B64 * LS;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int lrow = lane & 31, lk = lane >> 5, qi = wave >> 1, qj = wave & 1;
    const int blk = blockIdx.x;
    const int j0 = blk * kTrsmBlock;
    const int w = (n - j0) < kTrsmBlock ? (n - j0) : kTrsmBlock;
    const float* Ub = U + (long)j0 * ldu + j0;
    float* out = Uinv + (long)blk * kTrsmBlock * kTrsmBlock;
    if (tid < w && Ub[(long)tid * ldu + tid] == 0.f) atomicOr(flags, DQ_FLAG_SINGULAR);
    load_block64(Ub, ldu, w, 0, 0, B0, tid);
    tri_inv_upper_64<false>(B0, B1, tid);                   // B1 = A^-1
    store_block64(B1, out, w, 0, 0, tid);
    load_block64(Ub, ldu, w, B64, B64, B0, tid);
    tri_inv_upper_64<false>(B0, B2, tid);                   // B2 = C^-1
    store_block64(B2, out, w, B64, B64, tid);
    load_block64(Ub, ldu, w, 0, B64, B0, tid);              // B0 = B
    const f32x16 t = lds_mma<0>(B0, B2, nullptr, qi, qj, 0, 32 * (qj + 1), lrow, lk);
    __syncthreads();
    acc_to_lds(t, B0, qi, qj, lrow, lk);                    // B0 = B C^-1
    __syncthreads();
    const f32x16 x = lds_mma<0>(B1, B0, nullptr, qi, qj, 32 * qi, B64, lrow, lk);
#pragma unroll
    for (int v = 0; v < 16; ++v) {
        const int i = 32 * qi + 8 * (v >> 2) + 4 * lk + (v & 3), j = 32 * qj + lrow;
        out[(long)i * kTrsmBlock + B64 + j] = (i < w && B64 + j < w) ? -x[v] : 0.f;
        out[(long)(B64 + i) * kTrsmBlock + j] = 0.f;
    }
}

// out (n / kTrsmOuter blocks of kTrsmOuter x kTrsmOuter, row-major) = block diagonal of the kTrsmBlock inverses in
// `inv` (row-major kTrsmBlock x kTrsmBlock each), zero elsewhere
__global__ __launch_bounds__(256) void place_diag_blocks_kernel(const float* __restrict__ inv, float* __restrict__ out,
                                                                long total4) {
    constexpr int per = kTrsmOuter / kTrsmBlock;
    for (long e4 = (long)blockIdx.x * 256 + threadIdx.x; e4 < total4; e4 += (long)gridDim.x * 256) {
        const long e = e4 * 4;
        const long J = e / ((long)kTrsmOuter * kTrsmOuter);
        const int r = (int)((e / kTrsmOuter) % kTrsmOuter), c = (int)(e % kTrsmOuter);
        float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
        if (r / kTrsmBlock == c / kTrsmBlock)
            v = *reinterpret_cast<const float4*>(inv + ((J * per + r / kTrsmBlock) * kTrsmBlock + r % kTrsmBlock) * kTrsmBlock +
                                                 c % kTrsmBlock);
        *reinterpret_cast<float4*>(out + e) = v;
    }
}

__global__ __launch_bounds__(256) void axpy2d_kernel(float* __restrict__ Z, long ldz, const float* __restrict__ D,
                                                     long ldd, int n, float a) {
    const long total = (long)n * n;
    for (long e = (long)blockIdx.x * 256 + threadIdx.x; e < total; e += (long)gridDim.x * 256) {
        const int r = (int)(e / n), c = (int)(e % n);
        Z[(long)r * ldz + c] += a * D[(long)r * ldd + c];
    }
}

// Adam (bias-corrected) and heavy-ball momentum on the latent: HBM-bound elementwise passes over n x n matrices
// (Adam: 16 B read + 12 B written per element).  Row/column indexing because every matrix has its own leading
// dimension.
__global__ __launch_bounds__(256) void adam2d_kernel(float* __restrict__ Z, long ldz, const float* __restrict__ D, long ldd,
                                                     float* __restrict__ m, long ldm, float* __restrict__ v, long ldv, int rows,
                                                     int n, float lr, float beta1, float beta2, float omb1, float omb2, float eps, float c1,
                                                     float c2) {
    const int q = (n + 3) >> 2;
    const long total = (long)rows * q;
    for (long e = (long)blockIdx.x * 256 + threadIdx.x; e < total; e += (long)gridDim.x * 256) {
        const int r = (int)(e / q), c0 = (int)(e % q) << 2;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int c = c0 + j;
            if (c < n) {
                const float g = D[(long)r * ldd + c];
                const float mn = beta1 * m[(long)r * ldm + c] + omb1 * g;
                const float vn = beta2 * v[(long)r * ldv + c] + omb2 * g * g;
                m[(long)r * ldm + c] = mn;
                v[(long)r * ldv + c] = vn;
                Z[(long)r * ldz + c] -= lr * (mn * c1) / (sqrtf(vn * c2) + eps);
            }
        }
    }
}

__global__ __launch_bounds__(256) void momentum2d_kernel(float* __restrict__ Z, long ldz, const float* __restrict__ D,
                                                         long ldd, float* __restrict__ buf, long ldb, int n, float lr,
                                                         float mu) {
    const long total = (long)n * n;
    for (long e = (long)blockIdx.x * 256 + threadIdx.x; e < total; e += (long)gridDim.x * 256) {
        const int r = (int)(e / n), c = (int)(e % n);
        const float bn = mu * buf[(long)r * ldb + c] + D[(long)r * ldd + c];
        buf[(long)r * ldb + c] = bn;
        Z[(long)r * ldz + c] -= lr * bn;
    }
}

// ------------------------------------------------------------------------------------------------ stream hand-over
// (see HandOver in dq_internal.h)
__global__ void signal_kernel(unsigned long long* word, unsigned long long value) { handover_signal(word, value); }

__global__ void wait_kernel(const unsigned long long* word, unsigned long long value, long long limit_ticks,
                            unsigned* flags, unsigned long long* timed_out) {
    if (!handover_wait(word, value, limit_ticks, flags) && timed_out != nullptr)
        __hip_atomic_store(timed_out, 1ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

}  // namespace

int whip_grid(long rows, int cols) {
    const long chunks = rows * (long)((cols + 7) / 8);
    long g = (chunks + 255) / 256;
    constexpr int cap = 2048;   // workgroups that saturate HBM with eight 4 KiB pieces in flight each
    if (g > cap) g = cap;
    if (g < 1) g = 1;
    return (int)g;
}

hipError_t launch_whip(const float* Y, long ldy, int T, int n, float scale, void* dY, int dy_is_bf16, long lddy,
                       double* partials, int grid, hipStream_t s, int batch, long stride_y, long stride_dy) {
    if (batch < 1) return hipSuccess;
    // yvec: 0 scalar loads, 1 16-byte loads, 2 the flat path for dense rows, 3 the same with nontemporal loads
    // (Y beyond the 256 MiB last-level cache)
    constexpr long nt_bytes = 192L << 20;
    const bool big = (long)batch * T * n * 4 > nt_bytes;   // the whole batch streams through the cache
    const int yvec = ((reinterpret_cast<uintptr_t>(Y) & 15) == 0 && (ldy & 3) == 0) ? (big ? 3 : 2) : 0;
    if (dy_is_bf16) {
        const int dvec = ((reinterpret_cast<uintptr_t>(dY) & 15) == 0 && (lddy & 7) == 0) ? 1 : 0;
        hipLaunchKernelGGL((whip_kernel<true>), dim3(grid, batch), dim3(256), 0, s, Y, ldy, T, n, scale, dY, lddy,
                           partials, yvec, dvec, stride_y, stride_dy);
    } else {
        const int dvec = ((reinterpret_cast<uintptr_t>(dY) & 15) == 0 && (lddy & 3) == 0) ? 1 : 0;
        hipLaunchKernelGGL((whip_kernel<false>), dim3(grid, batch), dim3(256), 0, s, Y, ldy, T, n, scale, dY, lddy,
                           partials, yvec, dvec, stride_y, stride_dy);
    }
    return hipGetLastError();
}

hipError_t launch_loss_finish(const double* partials, int count, float scale, float* loss_dev, unsigned* flags,
                              hipStream_t s, int batch) {
    if (batch < 1) return hipSuccess;
    hipLaunchKernelGGL(loss_finish_kernel, dim3(batch), dim3(256), 0, s, partials, count, scale, loss_dev, flags);
    return hipGetLastError();
}

hipError_t launch_split_transpose_bf16(const float* R, long ldr, int n, bf16_t* RbT, long ldt, int koff,
                                       hipStream_t s) {
    if (n % 64 == 0 && koff == n && (ldr & 3) == 0 && (ldt & 7) == 0 && (reinterpret_cast<uintptr_t>(R) & 15) == 0 &&
        (reinterpret_cast<uintptr_t>(RbT) & 15) == 0)
        hipLaunchKernelGGL(split_transpose64_bf16_kernel, dim3(n / 64, n / 64), dim3(256), 0, s, R, ldr, RbT, ldt, koff);
    else
        hipLaunchKernelGGL(split_transpose_bf16_kernel, dim3((n + 31) / 32, (koff + 31) / 32), dim3(256), 0, s, R, ldr, n,
                           RbT, ldt, koff);
    return hipGetLastError();
}

hipError_t launch_split3_bf16(const float* A, long lda, int rows, int cols, bf16_t* out, long ldo, long plane, int transpose,
                              hipStream_t s) {
    if (rows <= 0 || cols <= 0) return hipSuccess;
    if (transpose) {
        if (rows % 64 == 0 && cols % 64 == 0 && (lda & 3) == 0 && (ldo & 7) == 0 && (plane & 7) == 0 &&
            (reinterpret_cast<uintptr_t>(A) & 15) == 0 && (reinterpret_cast<uintptr_t>(out) & 15) == 0)
            hipLaunchKernelGGL(split3_transpose64_bf16_kernel, dim3(cols / 64, rows / 64), dim3(256), 0, s, A, lda, out, ldo,
                               plane);
        else
            hipLaunchKernelGGL(split3_transpose_bf16_kernel, dim3((cols + 31) / 32, (rows + 31) / 32), dim3(256), 0, s, A,
                               lda, rows, cols, out, ldo, plane);
        return hipGetLastError();
    }
    if ((cols & 3) || (lda & 3) || (ldo & 3) || (plane & 3) || (reinterpret_cast<uintptr_t>(A) & 15) ||
        (reinterpret_cast<uintptr_t>(out) & 7))
        return hipErrorInvalidValue;
    const long total = (long)rows * (cols / 4);
    long blocks = (total + 255) / 256;
    if (blocks > 8192) blocks = 8192;
    hipLaunchKernelGGL(split3_bf16_kernel, dim3((unsigned)blocks), dim3(256), 0, s, A, lda, rows, cols / 4, out, ldo, plane);
    return hipGetLastError();
}

hipError_t launch_transpose_bf16(const bf16_t* src, long lds_, int rows, int cols, bf16_t* dst, long ldd,
                                 hipStream_t s) {
    if (rows <= 0 || cols <= 0) return hipSuccess;
    if ((rows & 63) || (cols & 63) || (lds_ & 7) || (ldd & 7) || lds_ < cols || ldd < rows ||
        (reinterpret_cast<uintptr_t>(src) & 15) || (reinterpret_cast<uintptr_t>(dst) & 15))
        return hipErrorInvalidValue;
    hipLaunchKernelGGL(transpose_bf16_kernel, dim3((rows >> 6) * (cols >> 6)), dim3(256), 0, s, src, lds_, rows, cols,
                       dst, ldd);
    return hipGetLastError();
}

hipError_t launch_hadamard_init(const float* sgn, int n, float* Z, long ldz, hipStream_t s) {
    long blocks = ((long)n * n + 255) / 256;
    if (blocks > 8192) blocks = 8192;
    const float c = (float)(1.0 / sqrt((double)n));
    hipLaunchKernelGGL(hadamard_init_kernel, dim3((unsigned)blocks), dim3(256), 0, s, sgn, n, c, Z, ldz);
    return hipGetLastError();
}

hipError_t launch_outlier_count(const float* Y, long ldy, int T, int n, float tau, unsigned long long* count,
                                hipStream_t s) {
    if (T <= 0 || n <= 0) return hipSuccess;
    long blocks = ((long)T * ((n + 3) / 4) + 255) / 256;
    if (blocks > 4096) blocks = 4096;
    hipLaunchKernelGGL(outlier_count_kernel, dim3((unsigned)blocks), dim3(256), 0, s, Y, ldy, T, n, tau, count);
    return hipGetLastError();
}

hipError_t launch_gather_rows(const void* src, long src_stride_bytes, int rows_in, const int* idx, int rows_out,
                              int row_bytes, void* out, long out_stride_bytes, unsigned* flags, hipStream_t s) {
    if (rows_out <= 0 || row_bytes <= 0) return hipSuccess;
    const int pieces = row_bytes >> 4;
    const int rpb = pieces >= 256 ? 1 : 256 / pieces;
    long blocks = ((long)rows_out + rpb - 1) / rpb;
    if (blocks > 8192) blocks = 8192;
    hipLaunchKernelGGL(gather_rows_kernel, dim3((unsigned)blocks), dim3(256), 0, s, static_cast<const char*>(src),
                       src_stride_bytes, rows_in, idx, rows_out, row_bytes, static_cast<char*>(out), out_stride_bytes,
                       rpb, flags);
    return hipGetLastError();
}

hipError_t launch_skew_lower(const float* B, long ldb, int n, float* P, long ldp, float* Mzero, long ldm,
                             hipStream_t s, int batch, long stride_b, long stride_p, long stride_m) {
    const int tb = (n + 31) / 32;
    if (batch < 1) return hipSuccess;
    const bool al = n % 64 == 0 && ((ldb | ldp | stride_b | stride_p) & 3) == 0 && (reinterpret_cast<uintptr_t>(B) & 15) == 0 &&
                    (reinterpret_cast<uintptr_t>(P) & 15) == 0 &&
                    (Mzero == nullptr || (((ldm | stride_m) & 3) == 0 && (reinterpret_cast<uintptr_t>(Mzero) & 15) == 0));
    if (al)
        hipLaunchKernelGGL(skew_lower64_kernel, dim3(n / 64, n / 64, batch), dim3(256), 0, s, B, ldb, P, ldp, Mzero, ldm,
                           stride_b, stride_p, stride_m);
    else
        hipLaunchKernelGGL(skew_lower_kernel, dim3(tb, tb, batch), dim3(256), 0, s, B, ldb, n, P, ldp, Mzero, ldm,
                           stride_b, stride_p, stride_m);
    return hipGetLastError();
}

hipError_t launch_trinv_blocks(const float* U, long ldu, int n, float* Uinv, unsigned* flags, hipStream_t s,
                               int batch, long stride_u, long stride_inv) {
    const int nb = (n + kTrsmBlock - 1) / kTrsmBlock;
    if (batch < 1) return hipSuccess;
    hipLaunchKernelGGL(trinv_blocks_kernel, dim3(nb, batch), dim3(NTHR), 0, s, U, ldu, n, Uinv, flags, stride_u,
                       stride_inv);
    return hipGetLastError();
}

hipError_t launch_place_diag_blocks(const float* inv, float* out, int n, hipStream_t s) {
    const long total4 = (long)n * kTrsmOuter / 4;
    long b = (total4 + 255) / 256;
    if (b > 4096) b = 4096;
    hipLaunchKernelGGL(place_diag_blocks_kernel, dim3((unsigned)b), dim3(256), 0, s, inv, out, total4);
    return hipGetLastError();
}

hipError_t launch_adam2d(float* Z, long ldz, const float* D, long ldd, float* m, long ldm, float* v, long ldv, int n,
                         float lr, float beta1, float beta2, float eps, float c1, float c2, hipStream_t s, int rows) {
    if (rows < 0) rows = n;
    // 1 - beta in double: in fp32 the difference 1 - 0.999 alone is off by 6e-5 relative
    const float omb1 = (float)(1.0 - (double)beta1), omb2 = (float)(1.0 - (double)beta2);
    long b = ((long)rows * ((n + 3) / 4) + 255) / 256;
    if (b > 8192) b = 8192;
    if (b < 1) return hipSuccess;
    hipLaunchKernelGGL(adam2d_kernel, dim3((unsigned)b), dim3(256), 0, s, Z, ldz, D, ldd, m, ldm, v, ldv, rows, n, lr, beta1,
                       beta2, omb1, omb2, eps, c1, c2);
    return hipGetLastError();
}

hipError_t launch_momentum2d(float* Z, long ldz, const float* D, long ldd, float* buf, long ldb, int n, float lr,
                             float mu, hipStream_t s) {
    long b = ((long)n * n + 255) / 256;
    if (b > 8192) b = 8192;
    hipLaunchKernelGGL(momentum2d_kernel, dim3((unsigned)b), dim3(256), 0, s, Z, ldz, D, ldd, buf, ldb, n, lr, mu);
    return hipGetLastError();
}

hipError_t launch_axpy2d(float* Z, long ldz, const float* D, long ldd, int n, float a, hipStream_t s) {
    long b = ((long)n * n + 255) / 256;
    if (b > 8192) b = 8192;
    hipLaunchKernelGGL(axpy2d_kernel, dim3((unsigned)b), dim3(256), 0, s, Z, ldz, D, ldd, n, a);
    return hipGetLastError();
}

hipError_t launch_stream_signal(unsigned long long* word, unsigned long long value, hipStream_t s) {
    hipLaunchKernelGGL(signal_kernel, dim3(1), dim3(1), 0, s, word, value);
    return hipGetLastError();
}

hipError_t launch_stream_wait(const unsigned long long* word, unsigned long long value, long limit_us, unsigned* flags,
                              unsigned long long* timed_out, hipStream_t s) {
    hipLaunchKernelGGL(wait_kernel, dim3(1), dim3(1), 0, s, word, value, (long long)limit_us * 100, flags, timed_out);
    return hipGetLastError();
}

}  // namespace dq
