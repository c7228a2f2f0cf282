// Batched path for many small rotations of size 128 (per-head rotations; the "heads" workload): every problem of a
// batch runs in the same launch.
//   * heads_qr_kernel: R, U = qr(Z) for one 128 x 128 latent per workgroup, entirely in LDS.  Alg. 2 as printed:
//     column by column, the reflector is applied to the trailing columns of the matrix and accumulated into the
//     orthogonal factor in the same step (A <- H A, Q <- Q H); the signs are then fixed so that diag(U) >= 0.
//   * heads_rlg_kernel: Alg. 1, rotation and loss steps, fused for bf16 activations.  A workgroup streams 64-token tiles of X once;
//     Y = X R (R as two bf16 planes held in registers), the Whip loss and its gradient (Eq. 4) and the tile's
//     contribution to G = X^T dY are formed on chip: Y and dY never reach HBM.
//   * heads_reduce_kernel: sums the per-workgroup partial G and loss.
// The derivative through the QR runs through the batched forms of the general kernels.
#include "dq_internal.h"
#include "dq_wave.h"


namespace dq {
namespace {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));

constexpr int HN = kHeadDim;     // matrix size of this path

__device__ __forceinline__ float wave_total(float v) {
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) v += __shfl_xor(v, o);
    return v;
}

__device__ __forceinline__ float lane_value(float v, int l) {
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), l));
}

__device__ __forceinline__ uint32_t to_bf16_rne(float f) {
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (u >> 16) | 0x40u;   // NaN stays NaN
    u += 0x7fffu + ((u >> 16) & 1u);
    return u >> 16;
}

// ------------------------------------------------------------------------------------------------ S1 + S2
// Alg. 2 with the unnormalised reflector vector: for column j, x = A[j:, j], beta = -sign(x_0) ||x||,
// u = x - beta e_0, H = I - gamma u u^T with gamma = 2 / u^T u  (the same reflection as the paper's normalised v);
// a column that is already zero below the diagonal gets H = I.
// 512 threads: four adjacent lanes ("item" i = tid / 4, part h = tid % 4) hold one column of A AND one row of Q in
// registers, lane part h owning the 4-row groups g with g % 4 == h of both.  Both get x <- x - gamma (u . x) u (the
// column only if it lies right of j), with ONE read of u from LDS for the two, the partial dot products of the four
// lanes meeting through DPP.  Columns are dealt to the items round-robin over the wavefronts (item i holds column
// 8 (i % 16) + i / 16), so that every wavefront keeps live columns to the end.  The owners of column j + 1 publish it in
// LDS at the end of step j, so a step needs one barrier; every wavefront forms the column norm itself.  Rows are handled
// in blocks of 16: blocks above the diagonal block are skipped (the block index is a template parameter, so register
// indices are static and a step runs straight-line code), the diagonal block substitutes u_0 for the raw pivot and
// zero above it.
constexpr int QS = 4;                   // lanes per column / row
constexpr int QB = 16;                  // rows per block = 4 groups, one per lane part
constexpr int NG = HN / 4 / QS;         // 4-row groups held by a thread (of its column and of its row)

__device__ __forceinline__ int item_column(int item) { return 8 * (item & 15) + (item >> 4); }
__device__ __forceinline__ int column_item(int c) { return 16 * (c & 7) + (c >> 3); }

// rows of this thread's k-th group: 4 * (k * QS + h) .. + 3
template <int JB>
__device__ __forceinline__ void publish_from(float* cb, const float (&x)[4 * NG], int h, int j) {
#pragma unroll
    for (int k = JB; k < NG; ++k) {
        const int i = 4 * (k * QS + h);
        float4 v = make_float4(x[4 * k], x[4 * k + 1], x[4 * k + 2], x[4 * k + 3]);
        if (k == JB) {   // diagonal block: entries above the diagonal are published as zero
            v.x = i >= j ? v.x : 0.f; v.y = i + 1 >= j ? v.y : 0.f; v.z = i + 2 >= j ? v.z : 0.f; v.w = i + 3 >= j ? v.w : 0.f;
        }
        *reinterpret_cast<float4*>(cb + i) = v;
    }
}

// x <- x - gamma (u . x) u for this thread's part of its column (if live) and of its row of Q, for block row JB = j / 16
// of the pivot; u is the published column with u_0 = uj in place of the raw pivot.
template <int JB>
__device__ __forceinline__ void reflect_from(const float* cb, float (&xc)[4 * NG], float (&xq)[4 * NG], bool col_live,
                                             int h, int j, float uj, float gamma) {
    float4 u[NG - JB];
#pragma unroll
    for (int k = JB; k < NG; ++k) u[k - JB] = *reinterpret_cast<const float4*>(cb + 4 * (k * QS + h));
    {   // diagonal block: the pivot entry becomes u_0 (the entries above it were published as zero)
        const int i = 4 * (JB * QS + h);
        float4& v = u[0];
        v.x = i == j ? uj : v.x; v.y = i + 1 == j ? uj : v.y; v.z = i + 2 == j ? uj : v.z; v.w = i + 3 == j ? uj : v.w;
    }
    // four independent partial sums per dot product: a lone dependent chain of 32 FMAs would set the pace of the step
    float c0 = 0.f, c1 = 0.f, c2 = 0.f, c3 = 0.f, q0 = 0.f, q1 = 0.f, q2 = 0.f, q3 = 0.f;
#pragma unroll
    for (int k = JB; k < NG; ++k) {
        const float4 v = u[k - JB];
        c0 += v.x * xc[4 * k]; c1 += v.y * xc[4 * k + 1]; c2 += v.z * xc[4 * k + 2]; c3 += v.w * xc[4 * k + 3];
        q0 += v.x * xq[4 * k]; q1 += v.y * xq[4 * k + 1]; q2 += v.z * xq[4 * k + 2]; q3 += v.w * xq[4 * k + 3];
    }
    float dc = (c0 + c1) + (c2 + c3), dq = (q0 + q1) + (q2 + q3);
    dc += lane_xor<1>(dc); dq += lane_xor<1>(dq);
    dc += lane_xor<2>(dc); dq += lane_xor<2>(dq);
    const float fc = col_live ? gamma * dc : 0.f;
    const float fq = gamma * dq;
#pragma unroll
    for (int k = JB; k < NG; ++k) {
        const float4 v = u[k - JB];
        xc[4 * k] -= fc * v.x; xc[4 * k + 1] -= fc * v.y; xc[4 * k + 2] -= fc * v.z; xc[4 * k + 3] -= fc * v.w;
        xq[4 * k] -= fq * v.x; xq[4 * k + 1] -= fq * v.y; xq[4 * k + 2] -= fq * v.z; xq[4 * k + 3] -= fq * v.w;
    }
}

#define DQ_BLOCK_SWITCH(jb, CALL)                                                                  \
    switch (jb) {                                                                                  \
        case 0: CALL(0); break;                                                                    \
        case 1: CALL(1); break;                                                                    \
        case 2: CALL(2); break;                                                                    \
        case 3: CALL(3); break;                                                                    \
        case 4: CALL(4); break;                                                                    \
        case 5: CALL(5); break;                                                                    \
        case 6: CALL(6); break;                                                                    \
        default: CALL(7); break;                                                                   \
    }

__global__ __launch_bounds__(HN * QS) void heads_qr_kernel(const float* __restrict__ Z, long ldz, long sz,
                                                           float* __restrict__ R, long ldr, long sr,
                                                           float* __restrict__ U, long ldu, long su,
                                                           unsigned* flags) {
    __shared__ __attribute__((aligned(16))) float cbuf[2][HN];
    __shared__ __attribute__((aligned(16))) float sgn[HN];
    const int tid = threadIdx.x, lane = tid & 63;
    const int item = tid / QS, h = tid % QS;
    const int col = item_column(item);   // this thread's column of A; its row of Q is `item`
    const float* Zp = Z + (long)blockIdx.x * sz;
    float xc[4 * NG], xq[4 * NG];
#pragma unroll
    for (int k = 0; k < NG; ++k)
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int i = 4 * (k * QS + h) + e;
            xc[4 * k + e] = Zp[(long)i * ldz + col];
            xq[4 * k + e] = (i == item) ? 1.f : 0.f;
        }
    float mydiag = 0.f;
    if (col == 0) publish_from<0>(cbuf[0], xc, h, 0);
    __syncthreads();
    for (int j = 0; j < HN; ++j) {
        const float* cb = cbuf[j & 1];
        // column norm below the pivot: DPP inside the rows of 16 lanes, then the four row sums through scalar registers
        const float a0 = cb[lane], a1 = cb[lane + 64];
        const float alpha = cb[j];
        float sr_ = (lane > j ? a0 * a0 : 0.f) + (lane + 64 > j ? a1 * a1 : 0.f);
        sr_ += lane_xor<1>(sr_);
        sr_ += lane_xor<2>(sr_);
        sr_ += lane_xor<4>(sr_);
        sr_ += lane_xor<8>(sr_);
        const float s = (lane_value(sr_, 0) + lane_value(sr_, 16)) + (lane_value(sr_, 32) + lane_value(sr_, 48));
        float beta = alpha;   // nothing below the pivot: H = I
        if (s != 0.f) {
            // hardware square root (1 ulp): beta only decides how exactly the column is annihilated; gamma is formed
            // from the u that is applied, so that H is orthogonal whatever the rounding of beta
            const float nrm = __builtin_amdgcn_sqrtf(alpha * alpha + s);
            beta = alpha >= 0.f ? -nrm : nrm;
            const float uj = alpha - beta;
            const float gamma = 2.f * __builtin_amdgcn_rcpf(s + uj * uj);
#define DQ_CALL(JB) reflect_from<JB>(cb, xc, xq, col > j, h, j, uj, gamma)
            DQ_BLOCK_SWITCH(j / QB, DQ_CALL)
#undef DQ_CALL
        }
        if (col == j) mydiag = beta;
        if (tid == 0) sgn[j] = beta >= 0.f ? 1.f : -1.f;
        if (col == j + 1) {
            float* nb = cbuf[(j + 1) & 1];
#define DQ_CALL(JB) publish_from<JB>(nb, xc, h, j + 1)
            DQ_BLOCK_SWITCH((j + 1) / QB, DQ_CALL)
#undef DQ_CALL
        }
        __syncthreads();
    }
    if (h == 0) {
        if (!(fabsf(mydiag) <= 3.0e38f)) atomicOr(flags, DQ_FLAG_NONFINITE);
        else if (mydiag == 0.f) atomicOr(flags, DQ_FLAG_SINGULAR);
    }
    if (U != nullptr) {   // U[i][c] = s_i A[i][c] above the diagonal, |diag| on it
        float* Up = U + (long)blockIdx.x * su;
#pragma unroll
        for (int k = 0; k < NG; ++k)
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int i = 4 * (k * QS + h) + e;
                Up[(long)i * ldu + col] = i < col ? sgn[i] * xc[4 * k + e] : (i == col ? fabsf(mydiag) : 0.f);
            }
    }
    {                     // R[r][c] = s_c Q[r][c]
        float* Rp = R + (long)blockIdx.x * sr + (long)item * ldr;
#pragma unroll
        for (int k = 0; k < NG; ++k) {
            const int c = 4 * (k * QS + h);
            const float4 sg = *reinterpret_cast<const float4*>(sgn + c);
            *reinterpret_cast<float4*>(Rp + c) =
                make_float4(xq[4 * k] * sg.x, xq[4 * k + 1] * sg.y, xq[4 * k + 2] * sg.z, xq[4 * k + 3] * sg.w);
        }
    }
}
#undef DQ_BLOCK_SWITCH

// ------------------------------------------------------------------------------------------------ S3 + S4 + S5
constexpr int TT = 64;            // tokens per tile
constexpr int XLD = HN + 8;       // halfwords per LDS row of an X tile (272 bytes: 16-byte rows, 4-bank skew)
constexpr int DLD = TT + 8;       // halfwords per LDS row of the transposed dY tile (144 bytes)

struct XRegs { uint4 q0, q1, q2, q3; };

// tile rows [t0, t0 + 64) of X (tokens >= tend read as zero): 16 threads per row, 16 bytes each
__device__ __forceinline__ XRegs fetch_x(const bf16_t* __restrict__ Xp, long ldx, int t0, int tend, int tid) {
    const int col = (tid & 15) * 8, row = t0 + (tid >> 4);
    const bf16_t* p = Xp + (long)row * ldx + col;
    XRegs r;
    r.q0 = r.q1 = r.q2 = r.q3 = make_uint4(0u, 0u, 0u, 0u);
    if (row < tend) r.q0 = *reinterpret_cast<const uint4*>(p);
    if (row + 16 < tend) r.q1 = *reinterpret_cast<const uint4*>(p + 16 * ldx);
    if (row + 32 < tend) r.q2 = *reinterpret_cast<const uint4*>(p + 32 * ldx);
    if (row + 48 < tend) r.q3 = *reinterpret_cast<const uint4*>(p + 48 * ldx);
    return r;
}
__device__ __forceinline__ void stash_x(bf16_t* Xs, int tid, const XRegs r) {
    bf16_t* p = Xs + (tid >> 4) * XLD + (tid & 15) * 8;
    *reinterpret_cast<uint4*>(p) = r.q0;
    *reinterpret_cast<uint4*>(p + 16 * XLD) = r.q1;
    *reinterpret_cast<uint4*>(p + 32 * XLD) = r.q2;
    *reinterpret_cast<uint4*>(p + 48 * XLD) = r.q3;
}

// One 64-token tile.  Wavefront w forms Y[:, 32w .. 32w+32) (two 32 x 32 accumulators), applies Eq. 4 and its
// derivative, leaves dY transposed in LDS; after the barrier it adds X_tile^T dY_tile to its 32 rows of G.
// Matrix-core operand layout (32x32x16 bf16): lane l supplies row/column (l & 31) and the 8 consecutive reduction
// indices 8 (l >> 5) ..; the 32 x 32 result holds row 8 (v >> 2) + 4 (l >> 5) + (v & 3), column (l & 31) in register v.
__device__ __forceinline__ void heads_tile(const bf16_t* Xs, bf16_t* dYs, const bf16x8 (&rhi)[8], const bf16x8 (&rlo)[8],
                                           f32x16 (&accG)[4], float& lsum, float scale, int wave, int lrow, int lk) {
    f32x16 y0, y1;
#pragma unroll
    for (int v = 0; v < 16; ++v) { y0[v] = 0.f; y1[v] = 0.f; }
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) {
        const bf16x8 a0 = *reinterpret_cast<const bf16x8*>(Xs + lrow * XLD + ks * 16 + lk * 8);
        const bf16x8 a1 = *reinterpret_cast<const bf16x8*>(Xs + (32 + lrow) * XLD + ks * 16 + lk * 8);
        y0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a0, rhi[ks], y0, 0, 0, 0);
        y1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a1, rhi[ks], y1, 0, 0, 0);
        y0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a0, rlo[ks], y0, 0, 0, 0);
        y1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a1, rlo[ks], y1, 0, 0, 0);
    }
    const int j = 32 * wave + lrow;
#pragma unroll
    for (int i = 0; i < 2; ++i) {
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            const int tok0 = i * 32 + 8 * g + 4 * lk;
            float d[4];
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const float y = i == 0 ? y0[4 * g + q] : y1[4 * g + q];
                const float ex = __expf(-fabsf(y));
                lsum += ex;   // rows past the end of the chunk hold y = 0 and add exactly 1 each: removed by the caller
                // scale * sgn(y) without comparisons: y * 2^126 has modulus >= 1 for every normal y (an overflow to
                // infinity is as good), so the median with -scale and +scale picks the signed bound; y = 0 stays 0
                const float sg = __builtin_amdgcn_fmed3f(y * 8.507059173e37f, -scale, scale);
                d[q] = -sg * ex;
            }
            const f32x2 d01 = {d[0], d[1]}, d23 = {d[2], d[3]};
            const bf16x2 b01 = __builtin_convertvector(d01, bf16x2), b23 = __builtin_convertvector(d23, bf16x2);
            *reinterpret_cast<uint2*>(dYs + j * DLD + tok0) =
                make_uint2(__builtin_bit_cast(uint32_t, b01), __builtin_bit_cast(uint32_t, b23));
        }
    }
    __syncthreads();
    const int ch = 32 * wave + lrow;   // this lane's row of G
#pragma unroll
    for (int kt = 0; kt < TT / 16; ++kt) {
        u32x4 au;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const uint32_t lo = Xs[(kt * 16 + lk * 8 + 2 * e) * XLD + ch];
            const uint32_t hi = Xs[(kt * 16 + lk * 8 + 2 * e + 1) * XLD + ch];
            au[e] = lo | (hi << 16);
        }
        const bf16x8 afr = __builtin_bit_cast(bf16x8, au);
#pragma unroll
        for (int jb = 0; jb < 4; ++jb) {
            const bf16x8 bfr = *reinterpret_cast<const bf16x8*>(dYs + (jb * 32 + lrow) * DLD + kt * 16 + lk * 8);
            accG[jb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(afr, bfr, accG[jb], 0, 0, 0);
        }
    }
}

// grid (splits, b): workgroup (s, p) handles tokens [s * chunk, min(T, (s+1) * chunk)) of problem p and writes its
// partial G to Gpart[(p * splits + s) * 128 * 128 ..] and its partial sum of exp(-|y|) to lpart[p * splits + s].
__global__ __launch_bounds__(256, 2) void heads_rlg_kernel(const bf16_t* __restrict__ X, long ldx, long sx, int T,
                                                        const float* __restrict__ R, long ldr, long sr, float scale,
                                                        float* __restrict__ Gpart, double* __restrict__ lpart,
                                                        int chunk) {
    __shared__ __attribute__((aligned(16))) bf16_t Xs[2][TT * XLD];
    __shared__ __attribute__((aligned(16))) bf16_t dYs[HN * DLD];
    __shared__ float wsum[4];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, lrow = lane & 31, lk = lane >> 5;
    const int split = blockIdx.x, prob = blockIdx.y, splits = gridDim.x;
    const bf16_t* Xp = X + (long)prob * sx;
    const float* Rp = R + (long)prob * sr;
    const int tbeg = split * chunk;
    const int tend = (tbeg + chunk < T) ? tbeg + chunk : T;
    const int ntiles = tend > tbeg ? (tend - tbeg + TT - 1) / TT : 0;

    // this wavefront's 32 columns of R as matrix-core operands: R = hi + lo, 16 mantissa bits
    bf16x8 rhi[8], rlo[8];
    {
        const int j = 32 * wave + lrow;
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) {
            u32x4 hi, lo;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const float r0 = Rp[(long)(ks * 16 + lk * 8 + 2 * e) * ldr + j];
                const float r1 = Rp[(long)(ks * 16 + lk * 8 + 2 * e + 1) * ldr + j];
                const uint32_t h0 = to_bf16_rne(r0), h1 = to_bf16_rne(r1);
                const uint32_t l0 = to_bf16_rne(r0 - __uint_as_float(h0 << 16));
                const uint32_t l1 = to_bf16_rne(r1 - __uint_as_float(h1 << 16));
                hi[e] = h0 | (h1 << 16);
                lo[e] = l0 | (l1 << 16);
            }
            rhi[ks] = __builtin_bit_cast(bf16x8, hi);
            rlo[ks] = __builtin_bit_cast(bf16x8, lo);
        }
    }

    f32x16 accG[4];
#pragma unroll
    for (int jb = 0; jb < 4; ++jb)
#pragma unroll
        for (int v = 0; v < 16; ++v) accG[jb][v] = 0.f;
    float lsum = 0.f;

    XRegs p0 = fetch_x(Xp, ldx, tbeg, tend, tid);
    XRegs p1 = fetch_x(Xp, ldx, tbeg + TT, tend, tid);
    stash_x(Xs[0], tid, p0);
    __syncthreads();
    for (int it = 0; it < ntiles; it += 2) {
        // tile `it` is in Xs[0], tile it+1 in p1; tile it+2 is requested into p0
        p0 = fetch_x(Xp, ldx, tbeg + (it + 2) * TT, tend, tid);
        heads_tile(Xs[0], dYs, rhi, rlo, accG, lsum, scale, wave, lrow, lk);
        stash_x(Xs[1], tid, p1);
        __syncthreads();
        if (it + 1 < ntiles) {
            p1 = fetch_x(Xp, ldx, tbeg + (it + 3) * TT, tend, tid);
            heads_tile(Xs[1], dYs, rhi, rlo, accG, lsum, scale, wave, lrow, lk);
        }
        stash_x(Xs[0], tid, p0);
        __syncthreads();
    }

    float* Gp = Gpart + ((long)prob * splits + split) * (HN * HN);
#pragma unroll
    for (int jb = 0; jb < 4; ++jb)
#pragma unroll
        for (int v = 0; v < 16; ++v)
            Gp[(32 * wave + 8 * (v >> 2) + 4 * lk + (v & 3)) * HN + jb * 32 + lrow] = accG[jb][v];
    lsum = wave_total(lsum);
    if (lane == 0) wsum[wave] = lsum;
    __syncthreads();
    if (tid == 0) {
        // the zero rows that pad the last tile contributed exp(0) = 1 per element
        const double pad = (double)(ntiles * TT - (tend > tbeg ? tend - tbeg : 0)) * HN;
        lpart[(long)prob * splits + split] =
            (double)wsum[0] + (double)wsum[1] + (double)wsum[2] + (double)wsum[3] - pad;
    }
}

// grid (16, b): G[p] = sum_s Gpart[p][s];  loss[p] = scale * sum_s lpart[p][s]
__global__ __launch_bounds__(256) void heads_reduce_kernel(const float* __restrict__ Gpart, const double* __restrict__ lpart,
                                                           int splits, float scale, float* __restrict__ G, long ldg,
                                                           long sg, float* __restrict__ loss, unsigned* flags) {
    const int prob = blockIdx.y;
    const int e = (blockIdx.x * 256 + threadIdx.x) * 4;   // 16 x 256 x 4 = 128 x 128
    const float* src = Gpart + (long)prob * splits * (HN * HN) + e;
    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
    for (int s = 0; s < splits; ++s) {
        const float4 v = *reinterpret_cast<const float4*>(src + (long)s * (HN * HN));
        acc.x += v.x; acc.y += v.y; acc.z += v.z; acc.w += v.w;
    }
    *reinterpret_cast<float4*>(G + (long)prob * sg + (long)(e >> 7) * ldg + (e & (HN - 1))) = acc;
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        double t = 0.0;
        for (int s = 0; s < splits; ++s) t += lpart[(long)prob * splits + s];
        const float Lf = (float)((double)scale * t);
        loss[prob] = Lf;
        if (!(fabsf(Lf) <= 3.0e38f)) atomicOr(flags, DQ_FLAG_NONFINITE);
    }
}

}  // namespace

hipError_t launch_heads_qr(int b, const float* Z, long ldz, long sz, float* R, long ldr, long sr, float* U, long ldu,
                           long su, unsigned* flags, hipStream_t s) {
    if (b < 1) return hipSuccess;
    hipLaunchKernelGGL(heads_qr_kernel, dim3(b), dim3(HN * QS), 0, s, Z, ldz, sz, R, ldr, sr, U, ldu, su, flags);
    return hipGetLastError();
}

int heads_splits(int T) { return (T + kHeadsChunk - 1) / kHeadsChunk; }

hipError_t launch_heads_rlg(int b, int T, const bf16_t* X, long ldx, long sx, const float* R, long ldr, long sr,
                            float scale, float* Gpart, double* lpart, float* G, long ldg, long sg, float* loss,
                            unsigned* flags, hipStream_t s) {
    if (b < 1) return hipSuccess;
    const int splits = heads_splits(T);
    hipLaunchKernelGGL(heads_rlg_kernel, dim3(splits, b), dim3(256), 0, s, X, ldx, sx, T, R, ldr, sr, scale, Gpart,
                       lpart, kHeadsChunk);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(heads_reduce_kernel, dim3(16, b), dim3(256), 0, s, Gpart, lpart, splits, scale, G, ldg, sg, loss,
                       flags);
    return hipGetLastError();
}

}  // namespace dq
