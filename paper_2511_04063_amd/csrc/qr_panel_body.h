// Device-side bodies of the one-workgroup Householder panel factorisation (Alg. 2 in LAPACK-style compact-WY form)
// and of the copy that unpacks its reflectors; shared by the stand-alone kernels and by the tall-panel route, which
// falls back to them inside its own kernel.
//
// Reflector convention: H = I - tau v v^T with v[0] = 1 implied, beta = -sign(alpha) ||x||,
// tau = (beta - alpha) / beta, v[1:] = x[1:] / (alpha - beta).  This is the same reflection as Alg. 2's
// normalised v = x + sign(x_1)||x|| e_1 (H = I - 2 v v^T / v^T v), stored without the normalisation.
#pragma once

#include "dq_internal.h"
#include "dq_wave.h"

namespace dq {

// One workgroup of NT threads factors an m x jb panel (m <= NT*Q).  The panel is processed in slices of
// SW columns; thread t keeps rows t, t+NT, ... of the current slice in registers.  Before a slice is
// factored, the reflector blocks of the earlier slices of the same panel are applied to it
// (left-looking), reading them back from `Vs`, a packed copy [slice][row][SW] with the unit diagonal and
// the zeros above it written out.  Every thread re-reads only rows it wrote itself.
template <int NT, int Q, int SW, int VCH>
__device__ __forceinline__ void qr_panel_body(float* __restrict__ A, long lda, int m, int jb, float* __restrict__ tau,
                                              float* Vs, float* __restrict__ tslices, unsigned* flags, int vec) {
    constexpr int NW = NT / 64;
    constexpr int MP = NT * Q;
    constexpr int NV2 = SW * SW;
    constexpr int NS = kPanel / SW;
    static_assert(NT >= kPanel, "the diagonal rows of a panel must belong to the first row set of each thread");
    __shared__ float red[2][NW][NV2];
    __shared__ float rowd[2][SW];
    __shared__ __attribute__((aligned(16))) float wsd[2][NW][SW];
    __shared__ float Wsh[NV2];
    __shared__ __attribute__((aligned(16))) float W2sh[NV2];
    __shared__ float Tsh[NS][NV2];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int ns = (jb + SW - 1) / SW;
    int par = 0;

    float a[Q][SW];

    for (int s = 0; s < ns; ++s) {
        const int col0 = s * SW;
        const int ncs = (jb - col0) < SW ? (jb - col0) : SW;

        // ---- load the slice
#pragma unroll
        for (int i = 0; i < Q; ++i) {
            const int r = tid + NT * i;
            const float* src = A + (long)r * lda + col0;
            if (r < m && vec && ncs == SW) {
#pragma unroll
                for (int c4 = 0; c4 < SW; c4 += 4) {
                    const float4 t4 = *reinterpret_cast<const float4*>(src + c4);
                    a[i][c4 + 0] = t4.x; a[i][c4 + 1] = t4.y; a[i][c4 + 2] = t4.z; a[i][c4 + 3] = t4.w;
                }
            } else {
#pragma unroll
                for (int c = 0; c < SW; ++c) a[i][c] = (r < m && c < ncs) ? src[c] : 0.f;
            }
        }

        // ---- apply the block reflectors of the earlier slices:  A_s -= V_p (T_p^T (V_p^T A_s))
        for (int p = 0; p < s; ++p) {
            // VCH rows of V_p are held at a time: all of them when they fit the register budget (one read of V_p),
            // otherwise V_p is streamed twice in chunks (projection, then update).
            float v[VCH][SW];
            float wacc[NV2];
#pragma unroll
            for (int e = 0; e < NV2; ++e) wacc[e] = 0.f;
#pragma unroll
            for (int i0 = 0; i0 < Q; i0 += VCH) {
#pragma unroll
                for (int ii = 0; ii < VCH; ++ii) {
                    const int r = tid + NT * (i0 + ii);
                    const float* src = Vs + ((long)p * MP + r) * SW;
#pragma unroll
                    for (int c4 = 0; c4 < SW; c4 += 4) {
                        const float4 t4 = *reinterpret_cast<const float4*>(src + c4);
                        v[ii][c4 + 0] = t4.x; v[ii][c4 + 1] = t4.y; v[ii][c4 + 2] = t4.z; v[ii][c4 + 3] = t4.w;
                    }
                }
#pragma unroll
                for (int ii = 0; ii < VCH; ++ii)
#pragma unroll
                    for (int cp = 0; cp < SW; ++cp)
#pragma unroll
                        for (int c = 0; c < SW; ++c) wacc[cp * SW + c] += v[ii][cp] * a[i0 + ii][c];
                if constexpr (VCH != Q) __builtin_amdgcn_sched_barrier(0);   // keep one chunk of V_p live at a time
            }
            const int idx = wave_reduce_multi<NV2>(wacc, lane);
            if (wave_reduce_writer<NV2>(lane)) red[0][wave][idx] = wacc[0];
            lds_barrier();
            if (tid < NV2) {
                float t = 0.f;
#pragma unroll
                for (int w = 0; w < NW; ++w) t += red[0][w][tid];
                Wsh[tid] = t;
            }
            lds_barrier();
            if (tid < NV2) {
                const int cp = tid / SW, c = tid % SW;
                float t = 0.f;
                for (int cq = 0; cq <= cp; ++cq) t += Tsh[p][cq * SW + cp] * Wsh[cq * SW + c];
                W2sh[tid] = t;
            }
            lds_barrier();
#pragma unroll
            for (int i0 = 0; i0 < Q; i0 += VCH) {
                if constexpr (VCH != Q) {
#pragma unroll
                    for (int ii = 0; ii < VCH; ++ii) {
                        const int r = tid + NT * (i0 + ii);
                        const float* src = Vs + ((long)p * MP + r) * SW;
#pragma unroll
                        for (int c4 = 0; c4 < SW; c4 += 4) {
                            const float4 t4 = *reinterpret_cast<const float4*>(src + c4);
                            v[ii][c4 + 0] = t4.x; v[ii][c4 + 1] = t4.y; v[ii][c4 + 2] = t4.z; v[ii][c4 + 3] = t4.w;
                        }
                    }
                }
#pragma unroll
                for (int cp = 0; cp < SW; ++cp) {
#pragma unroll
                    for (int c4 = 0; c4 < SW; c4 += 4) {
                        const float4 w4 = *reinterpret_cast<const float4*>(&W2sh[cp * SW + c4]);
#pragma unroll
                        for (int ii = 0; ii < VCH; ++ii) {
                            a[i0 + ii][c4 + 0] -= v[ii][cp] * w4.x;
                            a[i0 + ii][c4 + 1] -= v[ii][cp] * w4.y;
                            a[i0 + ii][c4 + 2] -= v[ii][cp] * w4.z;
                            a[i0 + ii][c4 + 3] -= v[ii][cp] * w4.w;
                        }
                    }
                }
                if constexpr (VCH != Q) __builtin_amdgcn_sched_barrier(0);
            }
        }

        // ---- factor the slice column by column
        if (tid < NV2) Tsh[s][tid] = 0.f;   // the slice's T factor is built in LDS by thread 0 (ordered by the
                                            // barrier of the first column step)
        float tau_l[SW];
#pragma unroll
        for (int c = 0; c < SW; ++c) {
            tau_l[c] = 0.f;
            if (c < ncs) {   // uniform over the workgroup
                const int d = col0 + c;
                float part[SW];
#pragma unroll
                for (int cp = 0; cp < SW; ++cp) part[cp] = 0.f;
                // branch-free: rows on or above the diagonal contribute zero
#pragma unroll
                for (int i = 0; i < Q; ++i) {
                    const int r = tid + NT * i;
                    const float ac = (r > d) ? a[i][c] : 0.f;
#pragma unroll
                    for (int cp = 0; cp < SW; ++cp) part[cp] += ac * a[i][cp];
                }
                if (tid == d) {   // d < kPanel <= NT: the diagonal row is row 0 of thread d; it publishes it
#pragma unroll
                    for (int cp = 0; cp < SW; ++cp) rowd[par][cp] = a[0][cp];
                }
                const int idx = wave_reduce_multi<SW>(part, lane);
                if (wave_reduce_writer<SW>(lane)) red[par][wave][idx] = part[0];
                lds_barrier();
                float sd[SW], rd[SW];
                if constexpr (NW * SW == 64) {
                    // one value per lane: lane l takes wavefront l / SW's partial of dot l % SW; the sum over the
                    // wavefronts is a 3-stage lane exchange; the SW totals go through a per-wavefront LDS row so that
                    // every lane can read all of them (same wavefront: no workgroup barrier needed)
                    float t = red[par][lane / SW][lane % SW];
                    t += lane_xor<8>(t);
                    t += lane_xor<16>(t);
                    t += lane_xor<32>(t);
                    if (lane < SW) wsd[par][wave][lane] = t;
                    __builtin_amdgcn_wave_barrier();
#pragma unroll
                    for (int cp = 0; cp < SW; ++cp) sd[cp] = wsd[par][wave][cp];
                } else {
#pragma unroll
                    for (int cp = 0; cp < SW; ++cp) {
                        float t = 0.f;
#pragma unroll
                        for (int w = 0; w < NW; ++w) t += red[par][w][cp];
                        sd[cp] = t;
                    }
                }
#pragma unroll
                for (int cp = 0; cp < SW; ++cp) rd[cp] = rowd[par][cp];
                par ^= 1;

                const float alpha = rd[c];
                const float xn2 = sd[c];
                float beta, tc, scale;
                if (xn2 == 0.f) {
                    beta = alpha; tc = 0.f; scale = 0.f;
                } else {
                    // hardware sqrt / reciprocal (1 ulp) with one Newton step on the reciprocals: the factorisation's
                    // backward error is set by the fp32 updates, not by the last bit of these three scalars
                    const float nrm = __builtin_amdgcn_sqrtf(alpha * alpha + xn2);
                    beta = alpha >= 0.f ? -nrm : nrm;
                    float rb = __builtin_amdgcn_rcpf(beta);
                    rb = rb * (2.f - beta * rb);
                    tc = (beta - alpha) * rb;
                    const float dd = alpha - beta;
                    float rs = __builtin_amdgcn_rcpf(dd);
                    scale = rs * (2.f - dd * rs);
                }
                if (tid == 0) {
                    if (!(fabsf(beta) <= 3.0e38f)) atomicOr(flags, DQ_FLAG_NONFINITE);
                    else if (beta == 0.f) atomicOr(flags, DQ_FLAG_SINGULAR);
                }
                tau_l[c] = tc;
                float w[SW];
#pragma unroll
                for (int cp = 0; cp < SW; ++cp) w[cp] = tc * (rd[cp] + scale * sd[cp]);
#pragma unroll
                for (int i = 0; i < Q; ++i) {
                    const int r = tid + NT * i;
                    const bool below = r > d, on = r == d;
                    const float vn = a[i][c] * scale;
                    const float f = below ? vn : (on ? 1.f : 0.f);   // the reflector's entry in this row
#pragma unroll
                    for (int cp = c + 1; cp < SW; ++cp) a[i][cp] -= w[cp] * f;
                    a[i][c] = below ? vn : (on ? beta : a[i][c]);
                }
                // column c of the slice's T:  T[0:c, c] = -tau * T[0:c, 0:c] * (V[:, 0:c]^T v_c),  T[c, c] = tau
                if (tid == 0) {
                    Tsh[s][c * SW + c] = tc;
#pragma unroll
                    for (int cp = 0; cp < c; ++cp) {
                        float t = 0.f;
#pragma unroll
                        for (int cq = cp; cq < c; ++cq) t += Tsh[s][cp * SW + cq] * (rd[cq] + scale * sd[cq]);
                        Tsh[s][cp * SW + c] = -tc * t;
                    }
                }
            }
        }

        // ---- store: in place (triangular factor on/above the diagonal, reflectors below) and the packed copy
#pragma unroll
        for (int c = 0; c < SW; ++c)
            if (tid == 64 + c && c < ncs) tau[col0 + c] = tau_l[c];   // every thread holds the same tau_l
#pragma unroll
        for (int i = 0; i < Q; ++i) {
            const int r = tid + NT * i;
            float* dst = A + (long)r * lda + col0;
            float pv[SW];
#pragma unroll
            for (int c = 0; c < SW; ++c) {
                const int d = col0 + c;
                pv[c] = (r < m && c < ncs) ? (r > d ? a[i][c] : (r == d ? 1.f : 0.f)) : 0.f;
            }
            // Rows below the panel's square top block hold reflector entries only; they reach A through
            // unpack_reflectors_kernel (full 256-byte rows) instead of 32-byte pieces from here.
            if (r < m && r < jb) {
                if (vec && ncs == SW) {
#pragma unroll
                    for (int c4 = 0; c4 < SW; c4 += 4)
                        *reinterpret_cast<float4*>(dst + c4) = make_float4(a[i][c4], a[i][c4 + 1], a[i][c4 + 2], a[i][c4 + 3]);
                } else {
#pragma unroll
                    for (int c = 0; c < SW; ++c)
                        if (c < ncs) dst[c] = a[i][c];
                }
            }
            float* vdst = Vs + ((long)s * MP + r) * SW;
#pragma unroll
            for (int c4 = 0; c4 < SW; c4 += 4)
                *reinterpret_cast<float4*>(vdst + c4) = make_float4(pv[c4], pv[c4 + 1], pv[c4 + 2], pv[c4 + 3]);
        }
        lds_barrier();
        if (tid < NV2) tslices[s * NV2 + tid] = Tsh[s][tid];
    }
}

// Copies rows jb..m-1 of a factored panel from the packed slice-major copy [slice][row][sw] into the matrix
// (row-major, lda): one 16-byte piece per thread, consecutive threads along a row.
__device__ __forceinline__ void unpack_reflectors_body(float* __restrict__ A, long lda, int m, int jb,
                                                       const float* __restrict__ Vs, int mp, int sw, int vec,
                                                       long first, long step) {
    const int c4n = (jb + 3) >> 2;                 // 16-byte pieces per row
    const long total = (long)(m - jb) * c4n;
    for (long e = first; e < total; e += step) {
        const int r = jb + (int)(e / c4n);
        const int c = (int)(e % c4n) << 2;
        const float4 v = *reinterpret_cast<const float4*>(Vs + ((long)(c / sw) * mp + r) * sw + (c % sw));
        float* dst = A + (long)r * lda + c;
        if (vec && c + 3 < jb) {
            *reinterpret_cast<float4*>(dst) = v;
        } else {
            if (c + 0 < jb) dst[0] = v.x;
            if (c + 1 < jb) dst[1] = v.y;
            if (c + 2 < jb) dst[2] = v.z;
            if (c + 3 < jb) dst[3] = v.w;
        }
    }
}

}  // namespace dq
