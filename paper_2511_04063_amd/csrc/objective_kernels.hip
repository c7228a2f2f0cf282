// Row-wise objectives that the paper compares with Eq. 4 (Sec. 4.1; Sec. 5, ablation of the optimisation objective):
// per-token variance, per-token kurtosis and the error of the per-token asymmetric uniform quantiser.  The paper names
// them and prints no formula; the definitions taken are stated at objective_rows_kernel.  Each is one pass over Y:
// a token row is held in the registers of the threads that own it, the row statistics are reduced over those threads,
// and dY leaves from the same registers, so HBM sees one read of Y and one write of dY like the Whip pass.
#include "dq_internal.h"
#include "dq_wave.h"

#include <climits>
#include <cstdlib>

namespace dq {
namespace {

typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));

constexpr int OBJ_VARIANCE = 1, OBJ_KURTOSIS = 2, OBJ_QUANT = 3;

__device__ __forceinline__ float wave_sum(float v) {
    v += lane_xor<1>(v); v += lane_xor<2>(v); v += lane_xor<4>(v);
    v += lane_xor<8>(v); v += lane_xor<16>(v); v += lane_xor<32>(v);
    return v;
}
__device__ __forceinline__ float wave_min(float v) {
    v = fminf(v, lane_xor<1>(v)); v = fminf(v, lane_xor<2>(v)); v = fminf(v, lane_xor<4>(v));
    v = fminf(v, lane_xor<8>(v)); v = fminf(v, lane_xor<16>(v)); v = fminf(v, lane_xor<32>(v));
    return v;
}
// the exchanges move bit patterns, so an integer travels as the float with its bits
template <int OFF>
__device__ __forceinline__ int lane_xor_int(int v) { return __float_as_int(lane_xor<OFF>(__int_as_float(v))); }
__device__ __forceinline__ int wave_min(int v) {
    v = min(v, lane_xor_int<1>(v)); v = min(v, lane_xor_int<2>(v)); v = min(v, lane_xor_int<4>(v));
    v = min(v, lane_xor_int<8>(v)); v = min(v, lane_xor_int<16>(v)); v = min(v, lane_xor_int<32>(v));
    return v;
}

// Totals over the TPR threads that share a row (TPR = 64: one wavefront, no LDS; TPR = 256: the workgroup, one barrier).
// `red` holds two sets of 4 x 8 words used alternately, so that consecutive calls need no second barrier.
struct RowReducer {
    float* red;
    int phase;
    template <int TPR, int NV>
    __device__ __forceinline__ void sum(float (&v)[NV], int tid) {
#pragma unroll
        for (int k = 0; k < NV; ++k) v[k] = wave_sum(v[k]);
        if constexpr (TPR > 64) {
            float* r = red + phase * 32;
            if ((tid & 63) == 0)
#pragma unroll
                for (int k = 0; k < NV; ++k) r[(tid >> 6) * 8 + k] = v[k];
            __syncthreads();
#pragma unroll
            for (int k = 0; k < NV; ++k) v[k] = (r[k] + r[8 + k]) + (r[16 + k] + r[24 + k]);
            phase ^= 1;
        }
    }
    // minimum of lo, minimum of nhi (the negated maximum)
    template <int TPR>
    __device__ __forceinline__ void min2(float& lo, float& nhi, int tid) {
        lo = wave_min(lo); nhi = wave_min(nhi);
        if constexpr (TPR > 64) {
            float* r = red + phase * 32;
            if ((tid & 63) == 0) { r[(tid >> 6) * 8] = lo; r[(tid >> 6) * 8 + 1] = nhi; }
            __syncthreads();
            lo = fminf(fminf(r[0], r[8]), fminf(r[16], r[24]));
            nhi = fminf(fminf(r[1], r[9]), fminf(r[17], r[25]));
            phase ^= 1;
        }
    }
    // two sums and two integer minima in one exchange
    template <int TPR>
    __device__ __forceinline__ void sum2_min2(float& s0, float& s1, int& i0, int& i1, int tid) {
        s0 = wave_sum(s0); s1 = wave_sum(s1); i0 = wave_min(i0); i1 = wave_min(i1);
        if constexpr (TPR > 64) {
            float* r = red + phase * 32;
            if ((tid & 63) == 0) {
                float* w = r + (tid >> 6) * 8;
                w[0] = s0; w[1] = s1; w[2] = __int_as_float(i0); w[3] = __int_as_float(i1);
            }
            __syncthreads();
            s0 = (r[0] + r[8]) + (r[16] + r[24]);
            s1 = (r[1] + r[9]) + (r[17] + r[25]);
            i0 = min(min(__float_as_int(r[2]), __float_as_int(r[10])), min(__float_as_int(r[18]), __float_as_int(r[26])));
            i1 = min(min(__float_as_int(r[3]), __float_as_int(r[11])), min(__float_as_int(r[19]), __float_as_int(r[27])));
            phase ^= 1;
        }
    }
};

// One token row y (n channels) per TPR threads, 4 V values per thread.  With c = `scale` (1/T or 1) and per row
//   mu = (1/n) sum_i y_i,  d_i = y_i - mu,  m_k = (1/n) sum_i d_i^k:
//   variance   loss_t = m2                    dY_i = c (2/n) d_i
//   kurtosis   loss_t = m4 / m2^2             dY_i = c (4/n) ((d_i^3 - m3) / m2^2 - m4 d_i / m2^3)     (0 if m2 = 0)
//   quant      lo = min y, hi = max y, delta = (hi - lo) / L, L = 2^bits - 1, s = 1 / delta,
//              q_i = rint((y_i - lo) * s) in fp32 (IEEE subtract, divide and multiply, ties to even),
//              e_i = y_i - (lo + delta q_i), loss_t = (1/n) sum e_i^2,
//              dY_j = c (2/n) (e_j - [j = jmin] sum_i e_i (1 - q_i / L) - [j = jmax] sum_i e_i q_i / L), the codes held
//              fixed and jmin / jmax the first positions of the minimum / maximum        (0 if delta = 0)
// partials[blockIdx.y * gridDim.x + blockIdx.x] receives the workgroup's sum of loss_t (the caller applies c).
// Element index of register (k, e): VEC (rows and strides of Y and dY 16-byte aligned, n % 4 == 0) 4 (k TPR + t) + e
// with 16-byte loads and 8- or 16-byte stores, else (4 k + e) TPR + t with 4-byte accesses.
// FULL: the row fills the registers exactly (n = 4 V TPR), no position needs a check (the quantiser, whose inner loop is
// the longest, gains 10 % from it and is the only objective instantiated that way).
// The row is transformed in place in its registers (y -> d or e -> dY), which keeps the kernel at 8 wavefronts per
// SIMD up to n = 8192.
template <int OBJ, int V, int TPR, bool BF16OUT, bool VEC, bool FULL>
__global__ __launch_bounds__(256) void objective_rows_kernel(const float* __restrict__ Y, long ldy, int T, int n,
                                                             float scale, float levels, void* __restrict__ dYv,
                                                             long lddy, double* __restrict__ partials, long sy,
                                                             long sdy) {
    __shared__ float red[64];
    __shared__ float tot[4];
    Y += (long)blockIdx.y * sy;
    if (dYv != nullptr) dYv = static_cast<char*>(dYv) + (long)blockIdx.y * sdy * (BF16OUT ? 2 : 4);
    const int tid = threadIdx.x;
    constexpr int RPW = 256 / TPR;                 // rows a workgroup holds at a time
    const int t = tid % TPR, sub = tid / TPR;
    RowReducer rr{red, 0};
    const float inv_n = 1.f / (float)n;
    float acc = 0.f;                               // this thread's share of sum_t loss_t
    // index of register 4 k + e in the row, and whether it lies inside the row
    auto at_index = [&](int k, int e) { return VEC ? 4 * (k * TPR + t) + e : (4 * k + e) * TPR + t; };
    auto load_row = [&](float (&r)[4 * V], long row) {
        const float* src = Y + row * ldy;
#pragma unroll
        for (int k = 0; k < V; ++k) {
            if constexpr (VEC) {
                const int i0 = 4 * (k * TPR + t);
                float4 q = make_float4(0.f, 0.f, 0.f, 0.f);
                if (FULL || i0 < n) q = *reinterpret_cast<const float4*>(src + i0);     // n % 4 == 0 on this route
                r[4 * k] = q.x; r[4 * k + 1] = q.y; r[4 * k + 2] = q.z; r[4 * k + 3] = q.w;
            } else {
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const int i = (4 * k + e) * TPR + t;
                    r[4 * k + e] = i < n ? src[i] : 0.f;
                }
            }
        }
    };
    const long row_step = (long)gridDim.x * RPW;
    long row = (long)blockIdx.x * RPW + sub;
    float x[4 * V], xn[4 * V];
    if (row < T) load_row(xn, row);
#pragma unroll 1
    for (; row < T; row += row_step) {
#pragma unroll
        for (int i = 0; i < 4 * V; ++i) x[i] = xn[i];
        if (row + row_step < T) load_row(xn, row + row_step);      // the next row travels while this one is worked on
        if constexpr (OBJ == OBJ_VARIANCE || OBJ == OBJ_KURTOSIS) {
            float s[1] = {0.f};
#pragma unroll
            for (int i = 0; i < 4 * V; ++i) s[0] += x[i];                       // entries outside the row are zero
            rr.sum<TPR, 1>(s, tid);
            const float mu = s[0] / (float)n;   // exact for a constant row whose sum is exact
            if constexpr (OBJ == OBJ_VARIANCE) {
                const float f = scale * 2.f * inv_n;
                float ss = 0.f;
#pragma unroll
                for (int k = 0; k < V; ++k)
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const float d = (FULL || at_index(k, e) < n) ? x[4 * k + e] - mu : 0.f;
                        ss += d * d;
                        x[4 * k + e] = f * d;
                    }
                acc += ss * inv_n;
            } else {
                float m[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int k = 0; k < V; ++k)
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const float d = (FULL || at_index(k, e) < n) ? x[4 * k + e] - mu : 0.f;
                        const float d2 = d * d;
                        x[4 * k + e] = d;
                        m[0] += d2; m[1] += d2 * d; m[2] += d2 * d2;
                    }
                rr.sum<TPR, 4>(m, tid);
                const float m2 = m[0] * inv_n, m3 = m[1] * inv_n, m4 = m[2] * inv_n;
                const bool flat = !(m2 > 0.f);
                const float r2 = flat ? 0.f : 1.f / (m2 * m2);
                const float kap = m4 * r2;
                if (t == 0) acc += kap;
                const float f = scale * 4.f * inv_n;
                const float a = f * r2, b = flat ? 0.f : f * kap / m2;          // f m4 / m2^3
#pragma unroll
                for (int k = 0; k < V; ++k)
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const float d = x[4 * k + e];
                        x[4 * k + e] = (FULL || at_index(k, e) < n) ? a * (d * d * d - m3) - b * d : 0.f;
                    }
            }
        } else {
            float lo = 3.0e38f, nhi = 3.0e38f;
#pragma unroll
            for (int k = 0; k < V; ++k)
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    if ((FULL || at_index(k, e) < n)) { lo = fminf(lo, x[4 * k + e]); nhi = fminf(nhi, -x[4 * k + e]); }
            const float own_lo = lo, own_nhi = nhi;
            rr.min2<TPR>(lo, nhi, tid);
            const float hi = -nhi;
            const float delta = __fdiv_rn(__fsub_rn(hi, lo), levels);
            const bool flat = !(delta > 0.f);
            const float inv_delta = flat ? 0.f : __fdiv_rn(1.f, delta);
            const float inv_l = 1.f / levels;
            // first position of the row minimum and maximum: only a wavefront that holds one of them looks for it
            int jmin = INT_MAX, jmax = INT_MAX;
            if (own_lo == lo || own_nhi == nhi) {
#pragma unroll
                for (int k = 0; k < V; ++k)
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const int i = at_index(k, e);
                        if ((FULL || i < n) && x[4 * k + e] == lo) jmin = min(jmin, i);
                        if ((FULL || i < n) && x[4 * k + e] == hi) jmax = min(jmax, i);
                    }
            }
            float se = 0.f, sq = 0.f, ss = 0.f;     // sums of e, e q, e^2
            const float f = scale * 2.f * inv_n;
#pragma unroll
            for (int k = 0; k < V; ++k)
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const float y = x[4 * k + e];
                    const bool in = (FULL || at_index(k, e) < n) && !flat;
                    // 0 <= (y - lo) / delta <= L up to one rounding, far from L + 1/2: the code needs no clamp
                    const float q = rintf(__fmul_rn(__fsub_rn(y, lo), inv_delta));
                    const float er = in ? y - (lo + delta * q) : 0.f;
                    ss += er * er;
                    se += er;
                    sq += er * q;
                    x[4 * k + e] = f * er;
                }
            acc += ss * inv_n;
            rr.sum2_min2<TPR>(se, sq, jmin, jmax, tid);
            // The two entries that also carry the dependence of lo and hi: every position of the minimum has e = 0 and
            // every position of the maximum the same e, so their values are known without looking them up.  Only a
            // wavefront that holds one of the two positions walks its registers.
            const float s1 = sq * inv_l, s0 = se - s1;      // sum e q / L and sum e (1 - q / L)
            const float q_hi = rintf(__fmul_rn(__fsub_rn(hi, lo), inv_delta));
            const float fix_lo = f * (0.f - s0);
            const float fix_hi = f * ((hi - (lo + delta * q_hi)) - s1);
            const bool mine_lo = !flat && jmin != INT_MAX && (VEC ? (jmin >> 2) % TPR : jmin % TPR) == t;
            const bool mine_hi = !flat && jmax != INT_MAX && (VEC ? (jmax >> 2) % TPR : jmax % TPR) == t;
            if (mine_lo || mine_hi) {
                // register position 4 k + e of a row index
                const int pos_lo = mine_lo ? (VEC ? 4 * ((jmin >> 2) / TPR) + (jmin & 3) : jmin / TPR) : -1;
                const int pos_hi = mine_hi ? (VEC ? 4 * ((jmax >> 2) / TPR) + (jmax & 3) : jmax / TPR) : -1;
#pragma unroll
                for (int p = 0; p < 4 * V; ++p) {
                    x[p] = p == pos_lo ? fix_lo : x[p];
                    x[p] = p == pos_hi ? fix_hi : x[p];
                }
            }
        }
        // dY from the registers, in the element order of the loads (a caller that wants the loss only passes no dY)
        if (dYv != nullptr)
#pragma unroll
        for (int k = 0; k < V; ++k) {
            if constexpr (VEC) {
                const int i0 = 4 * (k * TPR + t);
                if (i0 < n) {
                    if constexpr (BF16OUT) {
                        f32x2 a0 = {x[4 * k], x[4 * k + 1]}, a1 = {x[4 * k + 2], x[4 * k + 3]};
                        const bf16x2 b0 = __builtin_convertvector(a0, bf16x2), b1 = __builtin_convertvector(a1, bf16x2);
                        *reinterpret_cast<uint2*>(static_cast<bf16_t*>(dYv) + row * lddy + i0) =
                            make_uint2(__builtin_bit_cast(uint32_t, b0), __builtin_bit_cast(uint32_t, b1));
                    } else {
                        *reinterpret_cast<float4*>(static_cast<float*>(dYv) + row * lddy + i0) =
                            make_float4(x[4 * k], x[4 * k + 1], x[4 * k + 2], x[4 * k + 3]);
                    }
                }
            } else {
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const int i = at_index(k, e);
                    if (i < n) {
                        if constexpr (BF16OUT) {
                            const __bf16 hv = (__bf16)x[4 * k + e];
                            static_cast<bf16_t*>(dYv)[row * lddy + i] = __builtin_bit_cast(bf16_t, hv);
                        } else {
                            static_cast<float*>(dYv)[row * lddy + i] = x[4 * k + e];
                        }
                    }
                }
            }
        }
    }
    // workgroup total of the row losses (every wavefront arrives here: the row loop holds no barrier that a
    // wavefront could miss when TPR = 64, and all wavefronts of a row run the same trip count when TPR = 256)
    acc = wave_sum(acc);
    if ((tid & 63) == 0) tot[tid >> 6] = acc;
    __syncthreads();
    if (tid == 0)
        partials[(long)blockIdx.y * gridDim.x + blockIdx.x] = ((double)tot[0] + (double)tot[1]) + ((double)tot[2] + (double)tot[3]);
}

template <int OBJ, int V, int TPR>
hipError_t launch_rows(const float* Y, long ldy, int T, int n, float scale, float levels, void* dY, int dy_is_bf16,
                       long lddy, double* partials, int grid, int batch, long sy, long sdy, hipStream_t s) {
    const bool yvec = (reinterpret_cast<uintptr_t>(Y) & 15) == 0 && (ldy & 3) == 0 && (sy & 3) == 0 && (n & 3) == 0;
    const bool dvec = (reinterpret_cast<uintptr_t>(dY) & (dy_is_bf16 ? 7 : 15)) == 0 && (lddy & 3) == 0 && (sdy & 3) == 0;
    const dim3 g(grid, batch), b(256);
#define DQ_LAUNCH(BF, VEC, FULL)                                                                                  \
    hipLaunchKernelGGL((objective_rows_kernel<OBJ, V, TPR, BF, VEC, FULL>), g, b, 0, s, Y, ldy, T, n, scale, levels,  \
                       dY, lddy, partials, sy, sdy)
    if (OBJ == OBJ_QUANT && n == 4 * V * TPR && yvec && dvec) {
        if (dy_is_bf16) DQ_LAUNCH(true, true, (OBJ == OBJ_QUANT)); else DQ_LAUNCH(false, true, (OBJ == OBJ_QUANT));
    } else if (yvec && dvec) {
        if (dy_is_bf16) DQ_LAUNCH(true, true, false); else DQ_LAUNCH(false, true, false);
    } else {
        if (dy_is_bf16) DQ_LAUNCH(true, false, false); else DQ_LAUNCH(false, false, false);
    }
#undef DQ_LAUNCH
    return hipGetLastError();
}

template <int OBJ>
hipError_t launch_rows_shape(const float* Y, long ldy, int T, int n, float scale, float levels, void* dY,
                             int dy_is_bf16, long lddy, double* partials, int grid, int batch, long sy, long sdy,
                             hipStream_t s) {
#define DQ_ROWS(V, TPR) launch_rows<OBJ, V, TPR>(Y, ldy, T, n, scale, levels, dY, dy_is_bf16, lddy, partials, grid, batch, sy, sdy, s)
    if (n <= 256) return DQ_ROWS(1, 64);
    if (n <= 512) return DQ_ROWS(2, 64);
    if (n <= 1024) return DQ_ROWS(4, 64);
    if (n <= 2048) return DQ_ROWS(2, 256);
    if (n <= 3072) return DQ_ROWS(3, 256);
    if (n <= 4096) return DQ_ROWS(4, 256);
    if (n <= 5120) return DQ_ROWS(5, 256);
    if (n <= 6144) return DQ_ROWS(6, 256);
    if (n <= 8192) return DQ_ROWS(8, 256);
#undef DQ_ROWS
    return hipErrorInvalidValue;
}

}  // namespace

int objective_grid(int T, int n) {
    const int rpw = n <= 1024 ? 4 : 1;
    long g = ((long)T + rpw - 1) / rpw;
    // measured at T = 8192..16384: rows of n > 1024 (one workgroup per row) run best with about 1024 workgroups
    // that each walk several rows (the next row is fetched while one is worked on), short rows with 8192
    const long cap = n <= 1024 ? 8192L : 1024L;
    if (g > cap) g = cap;
    return (int)(g < 1 ? 1 : g);
}

hipError_t launch_objective(int objective, int bits, const float* Y, long ldy, int T, int n, float scale, void* dY,
                            int dy_is_bf16, long lddy, double* partials, int grid, hipStream_t s, int batch,
                            long stride_y, long stride_dy) {
    if (batch < 1 || T < 1) return hipSuccess;
    if (n < 1 || n > 8192 || bits < 1 || bits > 16) return hipErrorInvalidValue;
    const float levels = (float)((1 << bits) - 1);
    switch (objective) {
        case OBJ_VARIANCE:
            return launch_rows_shape<OBJ_VARIANCE>(Y, ldy, T, n, scale, levels, dY, dy_is_bf16, lddy, partials, grid,
                                                   batch, stride_y, stride_dy, s);
        case OBJ_KURTOSIS:
            return launch_rows_shape<OBJ_KURTOSIS>(Y, ldy, T, n, scale, levels, dY, dy_is_bf16, lddy, partials, grid,
                                                   batch, stride_y, stride_dy, s);
        case OBJ_QUANT:
            return launch_rows_shape<OBJ_QUANT>(Y, ldy, T, n, scale, levels, dY, dy_is_bf16, lddy, partials, grid,
                                                batch, stride_y, stride_dy, s);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace dq
