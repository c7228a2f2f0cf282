// fp32 GEMM on the CDNA4 matrix cores (v_mfma_f32_32x32x2_f32), LDS-staged, double-buffered.
//
//   C (M x N) = alpha * op(A) * op(B) + beta * C
//
// Workgroup: 256 threads = 4 wavefronts; workgroup tile 128 x 128 (64 x 256 for M <= 64, 256 x 64 for N <= 64),
// wavefront tile 64 x 64 = 2 x 2 MFMA tiles of 32 x 32; K step 16.  Both operand tiles live in LDS as [k][mn]
// (mn contiguous), so every MFMA operand fetch is a conflict-free 32-float row segment.
//
// MFMA 32x32x2 f32 lane layout (lane l of 64):  A operand a = A[m = l % 32][k = l / 32],
// B operand b = B[k = l / 32][n = l % 32], accumulator register v (0..15) holds
// D[m = 8*(v/4) + 4*(l/32) + v%4][n = l % 32].
//
// This kernel serves the trailing updates of the blocked Householder QR (Alg. 2 in compact-WY form),
// the accumulation of the orthogonal factor, the fp32 X @ R / X^T @ dY products and the three products
// of the derivative through Z = R U (the last step of Alg. 1).
#include "dq_internal.h"

namespace dq {

typedef float f32x16 __attribute__((ext_vector_type(16)));

namespace {


struct OperandView {
    const float* p; long ld;
    int row_lim, col_lim;   // storage rows / cols that may be read (others read as 0)
    int vec;                // 16-byte vector loads allowed
    int unit_lower_cols;    // storage columns < this get the unit-lower-trapezoid treatment (0: none)
};

__device__ __forceinline__ float4 load4_guarded(const OperandView& o, int sr, int sc) {
    float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
    if (sr < o.row_lim) {
        const float* q = o.p + (long)sr * o.ld + sc;
        if (o.vec && sc + 3 < o.col_lim) {
            v = *reinterpret_cast<const float4*>(q);
        } else {
            if (sc + 0 < o.col_lim) v.x = q[0];
            if (sc + 1 < o.col_lim) v.y = q[1];
            if (sc + 2 < o.col_lim) v.z = q[2];
            if (sc + 3 < o.col_lim) v.w = q[3];
        }
        if (o.unit_lower_cols > 0) {
            float* e = reinterpret_cast<float*>(&v);
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int c = sc + j;
                if (c < o.unit_lower_cols && c < o.col_lim) e[j] = (sr > c) ? e[j] : (sr == c ? 1.f : 0.f);
            }
        }
    }
    return v;
}

// KC = true : storage is (mn, k) with k contiguous  -> transposing store into LDS [k][mn]
// KC = false: storage is (k, mn) with mn contiguous -> straight 16-byte store
// ROWS = extent of the tile along mn, BK along k; every thread moves ROWS * BK / 1024 float4.
template <bool KC, int ROWS, int BK>
__device__ __forceinline__ void fetch_tile(const OperandView& o, int mn0, int k0, int tid,
                                           float4 (&frag)[ROWS * BK / 1024]) {
#pragma unroll
    for (int i = 0; i < ROWS * BK / 1024; ++i) {
        const int f = tid + 256 * i;
        if (KC) {
            const int r = f / (BK / 4), kq = (f % (BK / 4)) << 2;
            frag[i] = load4_guarded(o, mn0 + r, k0 + kq);
        } else {
            const int kr = f / (ROWS / 4), c4 = (f % (ROWS / 4)) << 2;
            frag[i] = load4_guarded(o, k0 + kr, mn0 + c4);
        }
    }
}

// The same for a tile that lies inside the operand with 16-byte aligned rows and needs no mask: plain 16-byte loads.
template <bool KC, int ROWS, int BK>
__device__ __forceinline__ void fetch_tile_inner(const float* __restrict__ p, long ld, int mn0, int k0, int tid,
                                                 float4 (&frag)[ROWS * BK / 1024]) {
#pragma unroll
    for (int i = 0; i < ROWS * BK / 1024; ++i) {
        const int f = tid + 256 * i;
        if (KC) {
            const int r = f / (BK / 4), kq = (f % (BK / 4)) << 2;
            frag[i] = *reinterpret_cast<const float4*>(p + (long)(mn0 + r) * ld + k0 + kq);
        } else {
            const int kr = f / (ROWS / 4), c4 = (f % (ROWS / 4)) << 2;
            frag[i] = *reinterpret_cast<const float4*>(p + (long)(k0 + kr) * ld + mn0 + c4);
        }
    }
}

template <bool KC, int ROWS, int BK>
__device__ __forceinline__ void stash_tile(float (*S)[ROWS + 4], int tid, const float4 (&frag)[ROWS * BK / 1024]) {
#pragma unroll
    for (int i = 0; i < ROWS * BK / 1024; ++i) {
        const int f = tid + 256 * i;
        if (KC) {
            const int r = f / (BK / 4), kq = (f % (BK / 4)) << 2;
            S[kq + 0][r] = frag[i].x;
            S[kq + 1][r] = frag[i].y;
            S[kq + 2][r] = frag[i].z;
            S[kq + 3][r] = frag[i].w;
        } else {
            const int kr = f / (ROWS / 4), c4 = (f % (ROWS / 4)) << 2;
            *reinterpret_cast<float4*>(&S[kr][c4]) = frag[i];
        }
    }
}

// BM x BN is the workgroup tile and WT the wavefront tile in units of 32 (wavefront tile 32*WT x 32*WT, four
// wavefronts): 128 x 128 (WT 2, waves 2 x 2), 64 x 256 (M <= 64) and 256 x 64 (N <= 64) for throughput, and
// 64 x 64 with WT 1 and a deeper K step for small latency-bound products that need many workgroups.
template <bool TA, bool TB, int BM, int BN, int WT, int BK>
__global__ __launch_bounds__(256) void gemm_f32_kernel(GemmF32 g, int tiles_m, int tiles_n, int avec, int bvec) {
    __shared__ __attribute__((aligned(16))) float As[2][BK][BM + 4];
    __shared__ __attribute__((aligned(16))) float Bs[2][BK][BN + 4];
    constexpr int WAVES_N = BN / (32 * WT);
    static_assert((BM / (32 * WT)) * WAVES_N == 4, "four wavefronts per workgroup");

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;

    // Workgroup ids are dealt round-robin to the 8 XCDs (each with its own L2): give each XCD a
    // contiguous run of tiles, and walk tiles in groups of 8 tile-rows so a run shares operand panels.
    const int nt = tiles_m * tiles_n;
    const int bid = blockIdx.x;
    const int q8 = nt >> 3, r8 = nt & 7;
    const int xcd = bid & 7;
    const int pid = xcd * q8 + (xcd < r8 ? xcd : r8) + (bid >> 3);
    const int group = 8 * tiles_n;
    const int gid = pid / group;
    const int first_m = gid * 8;
    const int gsz = (tiles_m - first_m) < 8 ? (tiles_m - first_m) : 8;
    int pid_m = first_m + (pid % group) % gsz;
    int pid_n = (pid % group) / gsz;
    if (g.b_strict_lower) {
        // The K loop of a tile starts at its column offset: tile columns are dealt out whole, longest first, so that
        // the long tiles do not start late and finish alone.
        pid_n = bid / tiles_m;
        pid_m = bid % tiles_m;
    }
    const int m0 = pid_m * BM, n0 = pid_n * BN;

    const int z = blockIdx.y;
    int kb = 0, ke = g.K;
    if (g.splits > 1) {
        kb = z * g.kchunk;
        ke = kb + g.kchunk < g.K ? kb + g.kchunk : g.K;
    }
    if (g.b_strict_lower) {
        const int lo = (n0 / BK) * BK;
        kb = kb > lo ? kb : lo;
    }

    OperandView oa, ob;
    const long bz = blockIdx.z;   // independent problem of a batched launch
    oa.p = g.A + bz * g.batch_a; oa.ld = g.lda; oa.vec = avec;
    oa.unit_lower_cols = g.a_unit_lower ? 0x7fffffff : 0;
    if (TA) { oa.row_lim = ke; oa.col_lim = g.M; } else { oa.row_lim = g.M; oa.col_lim = ke; }
    ob.p = g.B + bz * g.batch_b; ob.ld = g.ldb; ob.vec = bvec;
    ob.unit_lower_cols = g.b_unit_lower_cols;
    if (TB) { ob.row_lim = g.N; ob.col_lim = ke; } else { ob.row_lim = ke; ob.col_lim = g.N; }

    f32x16 acc[WT][WT];
#pragma unroll
    for (int i = 0; i < WT; ++i)
#pragma unroll
        for (int j = 0; j < WT; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    const int wm = (wave / WAVES_N) * 32 * WT, wn = (wave % WAVES_N) * 32 * WT;
    const int lrow = lane & 31, lk = lane >> 5;

    const int nk = ke > kb ? (ke - kb + BK - 1) / BK : 0;
    // A tile whose operand blocks and output block lie wholly inside the matrices, with aligned rows and out of reach
    // of the unit-lower masks, takes loaders and an epilogue without bounds checks: the checks cost more instructions
    // than the products of a short K loop.
    const bool inner = avec && bvec && m0 + BM <= g.M && n0 + BN <= g.N && ke > kb && (ke - kb) % BK == 0 &&
                       (!g.a_unit_lower || (!TA && m0 >= ke)) && (g.b_unit_lower_cols == 0 || (TB && n0 >= ke));
    float4 fa[BM * BK / 1024], fb[BN * BK / 1024];
    auto fetch_both = [&](int k0) {
        if (inner) {
            fetch_tile_inner<!TA, BM, BK>(oa.p, oa.ld, m0, k0, tid, fa);
            fetch_tile_inner<TB, BN, BK>(ob.p, ob.ld, n0, k0, tid, fb);
        } else {
            fetch_tile<!TA, BM, BK>(oa, m0, k0, tid, fa);
            fetch_tile<TB, BN, BK>(ob, n0, k0, tid, fb);
        }
    };
    if (nk > 0) {
        fetch_both(kb);
        stash_tile<!TA, BM, BK>(As[0], tid, fa);
        stash_tile<TB, BN, BK>(Bs[0], tid, fb);
    }
    __syncthreads();
    for (int kt = 0; kt < nk; ++kt) {
        const int cur = kt & 1;
        if (kt + 1 < nk) fetch_both(kb + (kt + 1) * BK);
#pragma unroll
        for (int kk = 0; kk < BK; kk += 2) {
            float a[WT], b[WT];
#pragma unroll
            for (int i = 0; i < WT; ++i) a[i] = As[cur][kk + lk][wm + i * 32 + lrow];
#pragma unroll
            for (int j = 0; j < WT; ++j) b[j] = Bs[cur][kk + lk][wn + j * 32 + lrow];
#pragma unroll
            for (int i = 0; i < WT; ++i)
#pragma unroll
                for (int j = 0; j < WT; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[i], b[j], acc[i][j], 0, 0, 0);
        }
        if (kt + 1 < nk) {
            stash_tile<!TA, BM, BK>(As[cur ^ 1], tid, fa);
            stash_tile<TB, BN, BK>(Bs[cur ^ 1], tid, fb);
        }
        __syncthreads();
    }

    float* C = g.C + bz * g.batch_c + (long)z * g.split_stride;
    // the scale of the product may also carry a factor that only the device knows (a step size formed by a kernel)
    const float alpha = g.alpha_dev != nullptr ? g.alpha * *g.alpha_dev : g.alpha, beta = g.beta;
    if (inner) {
        // one base pointer per 32 x 32 block and constant row offsets from it
        float* cb[WT][WT];
#pragma unroll
        for (int i = 0; i < WT; ++i)
#pragma unroll
            for (int j = 0; j < WT; ++j) cb[i][j] = C + (long)(m0 + wm + i * 32 + 4 * lk) * g.ldc + n0 + wn + j * 32 + lrow;
        if (beta != 0.f) {
            float cin[WT][WT][16];
#pragma unroll
            for (int i = 0; i < WT; ++i)
#pragma unroll
                for (int j = 0; j < WT; ++j)
#pragma unroll
                    for (int v = 0; v < 16; ++v) cin[i][j][v] = cb[i][j][(long)(8 * (v >> 2) + (v & 3)) * g.ldc];
#pragma unroll
            for (int i = 0; i < WT; ++i)
#pragma unroll
                for (int j = 0; j < WT; ++j)
#pragma unroll
                    for (int v = 0; v < 16; ++v) acc[i][j][v] = alpha * acc[i][j][v] + beta * cin[i][j][v];
        } else {
#pragma unroll
            for (int i = 0; i < WT; ++i)
#pragma unroll
                for (int j = 0; j < WT; ++j)
#pragma unroll
                    for (int v = 0; v < 16; ++v) acc[i][j][v] *= alpha;
        }
#pragma unroll
        for (int i = 0; i < WT; ++i)
#pragma unroll
            for (int j = 0; j < WT; ++j)
#pragma unroll
                for (int v = 0; v < 16; ++v) cb[i][j][(long)(8 * (v >> 2) + (v & 3)) * g.ldc] = acc[i][j][v];
    } else {
    // All reads of C are issued before the first write: interleaved they would serialise on possible aliasing and
    // expose one memory round trip per element.
    if (beta != 0.f) {
#pragma unroll
        for (int i = 0; i < WT; ++i) {
#pragma unroll
            for (int j = 0; j < WT; ++j) {
                const int col = n0 + wn + j * 32 + lrow;
                float cin[16];
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int row = m0 + wm + i * 32 + 8 * (v >> 2) + 4 * lk + (v & 3);
                    cin[v] = (row < g.M && col < g.N) ? C[(long)row * g.ldc + col] : 0.f;
                }
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[i][j][v] = alpha * acc[i][j][v] + beta * cin[v];
            }
        }
    } else {
#pragma unroll
        for (int i = 0; i < WT; ++i)
#pragma unroll
            for (int j = 0; j < WT; ++j)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[i][j][v] *= alpha;
    }
#pragma unroll
    for (int i = 0; i < WT; ++i) {
#pragma unroll
        for (int j = 0; j < WT; ++j) {
            const int col = n0 + wn + j * 32 + lrow;
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int row = m0 + wm + i * 32 + 8 * (v >> 2) + 4 * lk + (v & 3);
                if (row < g.M && col < g.N) C[(long)row * g.ldc + col] = acc[i][j][v];
            }
        }
    }
    }   // guarded epilogue
}

__global__ __launch_bounds__(256) void splitk_reduce_kernel(const float* __restrict__ part, int splits, long stride,
                                                            long ldp, int rows, int cols, float alpha, float beta,
                                                            float* __restrict__ out, long ldo) {
    const long total = (long)rows * cols;
    for (long e = (long)blockIdx.x * blockDim.x + threadIdx.x; e < total; e += (long)gridDim.x * blockDim.x) {
        const int r = (int)(e / cols), c = (int)(e % cols);
        float s = 0.f;
        const float* q = part + (long)r * ldp + c;
        int zz = 0;
        for (; zz + 8 <= splits; zz += 8) {     // eight independent loads in flight
            float t[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) t[u] = q[(long)(zz + u) * stride];
#pragma unroll
            for (int u = 0; u < 8; ++u) s += t[u];
        }
        for (; zz < splits; ++zz) s += q[(long)zz * stride];
        float* o = out + (long)r * ldo + c;
        float v = alpha * s;
        if (beta != 0.f) v += beta * *o;
        *o = v;
    }
}

// The same sum for rows that can be read 16 bytes at a time (cols, ldp, stride, ldo multiples of 4, aligned bases):
// one row piece of four columns per thread, no division per element, four layers in flight.
__global__ __launch_bounds__(256) void splitk_reduce4_kernel(const float* __restrict__ part, int splits, long stride,
                                                             long ldp, int rows, int cols4, float alpha, float beta,
                                                             float* __restrict__ out, long ldo) {
    const int c4 = blockIdx.x * 64 + (threadIdx.x & 63);
    if (c4 >= cols4) return;
    for (int r = blockIdx.y * 4 + (threadIdx.x >> 6); r < rows; r += gridDim.y * 4) {
        const float4* q = reinterpret_cast<const float4*>(part + (long)r * ldp) + c4;
        const long st4 = stride >> 2;
        float4 s = make_float4(0.f, 0.f, 0.f, 0.f);
        int zz = 0;
        for (; zz + 4 <= splits; zz += 4) {
            float4 t[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) t[u] = q[(long)(zz + u) * st4];
#pragma unroll
            for (int u = 0; u < 4; ++u) { s.x += t[u].x; s.y += t[u].y; s.z += t[u].z; s.w += t[u].w; }
        }
        for (; zz < splits; ++zz) {
            const float4 t = q[(long)zz * st4];
            s.x += t.x; s.y += t.y; s.z += t.z; s.w += t.w;
        }
        float4* o = reinterpret_cast<float4*>(out + (long)r * ldo) + c4;
        float4 v = make_float4(alpha * s.x, alpha * s.y, alpha * s.z, alpha * s.w);
        if (beta != 0.f) {
            const float4 old = *o;
            v.x += beta * old.x; v.y += beta * old.y; v.z += beta * old.z; v.w += beta * old.w;
        }
        *o = v;
    }
}

}  // namespace

template <int BM, int BN, int WT, int BK>
static hipError_t launch_gemm_f32_tile(const GemmF32& g, hipStream_t s) {
    const int tiles_m = (g.M + BM - 1) / BM, tiles_n = (g.N + BN - 1) / BN;
    const int avec = ((reinterpret_cast<uintptr_t>(g.A) & 15) == 0 && (g.lda & 3) == 0 && (g.batch_a & 3) == 0) ? 1 : 0;
    const int bvec = ((reinterpret_cast<uintptr_t>(g.B) & 15) == 0 && (g.ldb & 3) == 0 && (g.batch_b & 3) == 0) ? 1 : 0;
    dim3 grid(tiles_m * tiles_n, g.splits > 1 ? g.splits : 1, g.batch > 1 ? g.batch : 1);
    dim3 block(256, 1, 1);
    if (g.ta && g.tb)
        hipLaunchKernelGGL((gemm_f32_kernel<true, true, BM, BN, WT, BK>), grid, block, 0, s, g, tiles_m, tiles_n, avec, bvec);
    else if (g.ta)
        hipLaunchKernelGGL((gemm_f32_kernel<true, false, BM, BN, WT, BK>), grid, block, 0, s, g, tiles_m, tiles_n, avec, bvec);
    else if (g.tb)
        hipLaunchKernelGGL((gemm_f32_kernel<false, true, BM, BN, WT, BK>), grid, block, 0, s, g, tiles_m, tiles_n, avec, bvec);
    else
        hipLaunchKernelGGL((gemm_f32_kernel<false, false, BM, BN, WT, BK>), grid, block, 0, s, g, tiles_m, tiles_n, avec, bvec);
    return hipGetLastError();
}

// 1 = 64 x 256 tile, 2 = 256 x 64, 3 = 64 x 64 (many small workgroups), 0 = 128 x 128
static int gemm_f32_config(int M, int N, int splits) {
    const long big_tiles = (long)((M + 127) / 128) * ((N + 127) / 128) * (splits > 1 ? splits : 1);
    if (big_tiles < 96 && N <= 128) return 3;   // few output tiles: 64 x 64 tiles give more workgroups
    if (M <= 64 && N > 64) return 1;
    if (big_tiles < 96) return 3;      // would leave most compute units idle: use 64 x 64 tiles
    if (N <= 64) return 2;
    return 0;
}

int gemm_f32_tile_n(int M, int N) { return N <= 128 ? 64 : ((M <= 64) ? 256 : 128); }

hipError_t launch_gemm_f32(const GemmF32& g, hipStream_t s) {
    if (g.M <= 0 || g.N <= 0) return hipSuccess;
    switch (g.cfg >= 0 ? g.cfg : gemm_f32_config(g.M, g.N, g.splits)) {
        case 1: return launch_gemm_f32_tile<64, 256, 2, 16>(g, s);
        case 2: return launch_gemm_f32_tile<256, 64, 2, 16>(g, s);
        case 3: return launch_gemm_f32_tile<64, 64, 1, 32>(g, s);
        default: return launch_gemm_f32_tile<128, 128, 2, 16>(g, s);
    }
}

hipError_t launch_splitk_reduce(const float* part, int splits, long stride, long ldp, int rows, int cols,
                                float alpha, float beta, float* out, long ldo, hipStream_t s) {
    if (rows <= 0 || cols <= 0) return hipSuccess;
    if ((cols & 3) == 0 && (ldp & 3) == 0 && (stride & 3) == 0 && (ldo & 3) == 0 &&
        (reinterpret_cast<uintptr_t>(part) & 15) == 0 && (reinterpret_cast<uintptr_t>(out) & 15) == 0) {
        const int cols4 = cols >> 2;
        int gy = (rows + 3) / 4;
        if (gy > 2048) gy = 2048;
        hipLaunchKernelGGL(splitk_reduce4_kernel, dim3((cols4 + 63) / 64, gy), dim3(256), 0, s, part, splits, stride,
                           ldp, rows, cols4, alpha, beta, out, ldo);
        return hipGetLastError();
    }
    const long total = (long)rows * cols;
    long blocks = (total + 255) / 256;
    if (blocks > 4096) blocks = 4096;
    hipLaunchKernelGGL(splitk_reduce_kernel, dim3((unsigned)blocks), dim3(256), 0, s, part, splits, stride, ldp,
                       rows, cols, alpha, beta, out, ldo);
    return hipGetLastError();
}

}  // namespace dq
