// Wavefront-level helpers shared by the panel-factorisation kernels (device code only).
#pragma once

#include <hip/hip_runtime.h>

namespace dq {
namespace {

// Value of lane (l ^ OFF) for OFF in {1, 2, 4, 8, 16, 32}.  Distances inside a row of 16 lanes use DPP
// (quad_perm for 1 and 2, row_ror:8 for 8, a row_shl:4 / row_shr:4 pair masked by bank for 4), distance 16 uses
// ds_swizzle in bit mode, distance 32 the LDS permute.
template <int OFF>
__device__ __forceinline__ float lane_xor(float v) {
    const int x = __float_as_int(v);
    int r;
    if constexpr (OFF == 1) {
        r = __builtin_amdgcn_update_dpp(x, x, 0xB1, 0xF, 0xF, false);          // quad_perm:[1,0,3,2]
    } else if constexpr (OFF == 2) {
        r = __builtin_amdgcn_update_dpp(x, x, 0x4E, 0xF, 0xF, false);          // quad_perm:[2,3,0,1]
    } else if constexpr (OFF == 8) {
        r = __builtin_amdgcn_update_dpp(x, x, 0x128, 0xF, 0xF, false);         // row_ror:8
    } else if constexpr (OFF == 4) {
        r = __builtin_amdgcn_update_dpp(x, x, 0x104, 0xF, 0x5, false);         // row_shl:4 into banks 0 and 2
        r = __builtin_amdgcn_update_dpp(r, x, 0x114, 0xF, 0xA, false);         // row_shr:4 into banks 1 and 3
    } else if constexpr (OFF == 16) {
        r = __builtin_amdgcn_ds_swizzle(x, 0x401F);                            // bit mode: xor 16
    } else {
        return __shfl_xor(v, 32);
    }
    return __int_as_float(r);
}

// Sum NV per-lane values over the 64 lanes of a wavefront with a halving butterfly: after the call
// v[0] of every lane holds the wavefront total of the value whose index is returned.  Stage k pairs lanes that
// differ in bit kStageOff[k]; the stages that move the most values come first and use the cheapest exchanges.
// Written as a compile-time recursion so that every register index is static.
template <int S> struct StageOff;
template <> struct StageOff<0> { static constexpr int v = 1; };
template <> struct StageOff<1> { static constexpr int v = 2; };
template <> struct StageOff<2> { static constexpr int v = 8; };
template <> struct StageOff<3> { static constexpr int v = 4; };
template <> struct StageOff<4> { static constexpr int v = 16; };
template <> struct StageOff<5> { static constexpr int v = 32; };

template <int NV, int N, int S>
__device__ __forceinline__ int wave_reduce_stage(float (&v)[NV], int lane) {
    if constexpr (S >= 6) {
        return 0;
    } else {
        constexpr int OFF = StageOff<S>::v;
        if constexpr (N > 1) {
            constexpr int half = N / 2;
            const bool up = (lane & OFF) != 0;
#pragma unroll
            for (int k = 0; k < half; ++k) {
                const float keep = up ? v[k + half] : v[k];
                const float send = up ? v[k] : v[k + half];
                v[k] = keep + lane_xor<OFF>(send);
            }
            return (up ? half : 0) + wave_reduce_stage<NV, half, S + 1>(v, lane);
        } else {
            v[0] += lane_xor<OFF>(v[0]);
            return wave_reduce_stage<NV, 1, S + 1>(v, lane);
        }
    }
}
// Lanes whose bits of the non-halving stages are all zero hold one copy of each total: they are the writers.
template <int NV>
__device__ __forceinline__ bool wave_reduce_writer(int lane) {
    int mask = 0, n = NV;
    if (n > 1) n >>= 1; else mask |= 1;
    if (n > 1) n >>= 1; else mask |= 2;
    if (n > 1) n >>= 1; else mask |= 8;
    if (n > 1) n >>= 1; else mask |= 4;
    if (n > 1) n >>= 1; else mask |= 16;
    if (n > 1) n >>= 1; else mask |= 32;
    return (lane & mask) == 0;
}
template <int NV>
__device__ __forceinline__ int wave_reduce_multi(float (&v)[NV], int lane) {
    static_assert(NV >= 1 && NV <= 64 && (NV & (NV - 1)) == 0, "NV must be a power of two <= 64");
    return wave_reduce_stage<NV, NV, 0>(v, lane);
}

// Workgroup barrier that orders LDS traffic only: it waits for this wavefront's outstanding LDS operations
// (lgkmcnt) but not for its global stores (vmcnt), which __syncthreads() would also drain.  The panel kernel
// exchanges data between threads through LDS alone; global memory is only re-read by the thread that wrote it.
__device__ __forceinline__ void lds_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }

}  // namespace
}  // namespace dq
