// bf16 x bf16 -> fp32 GEMM on the CDNA4 matrix cores (v_mfma_f32_32x32x16_bf16), LDS-staged,
// double-buffered:   C (M x N, fp32) = op(A) * op(B).
//
// Serves the two large products of Alg. 1:  O = X @ R (its rotation step; X bf16, R split into two bf16 planes hi + lo
// and stored transposed so that both operands are k-contiguous) and G = X^T @ dY (the chain rule to R; both operands
// are stored with the reduction dimension, the tokens, as rows, and are transposed on their way into LDS).
//
// Workgroup: 256 threads = 2 x 2 wavefronts; tile 128 x 128 x 32; wavefront tile 64 x 64 = 2 x 2 MFMA tiles.
// LDS keeps both operands as [mn][k] with k contiguous (row stride 40 halfwords = 80 bytes).
//
// MFMA 32x32x16 bf16 lane layout (lane l of 64): the A operand holds 8 consecutive k of row m = l % 32, the
// B operand 8 consecutive k of column n = l % 32, both for k group l / 32; accumulator register v holds
// D[m = 8*(v/4) + 4*(l/32) + v%4][n = l % 32].  Both operands are fetched with the same k assignment, so
// only the m / n / D mappings matter for correctness.
#include <stdlib.h>

#include <utility>

#include "dq_internal.h"

namespace dq {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

namespace {

constexpr int BM = 128, BN = 128, BK = 32;
constexpr int LDH = BK + 8;   // LDS row stride in halfwords

struct OperandViewH {
    const bf16_t* p; long ld;
    int row_lim, col_lim;
    int vec;                  // 16-byte loads allowed (k-contiguous path)
};

union Frag {
    uint4 q[2];
    uint32_t w[8];
};

// k-contiguous storage (mn, k): two 16-byte chunks per thread
__device__ __forceinline__ void fetch_kc(const OperandViewH& o, int mn0, int k0, int tid, Frag& fr) {
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int f = tid + 256 * i;
        const int sr = mn0 + (f >> 2), sc = k0 + ((f & 3) << 3);
        uint4 v = make_uint4(0u, 0u, 0u, 0u);
        if (sr < o.row_lim) {
            const bf16_t* q = o.p + (long)sr * o.ld + sc;
            if (o.vec && sc + 7 < o.col_lim) {
                v = *reinterpret_cast<const uint4*>(q);
            } else {
                uint32_t e[8];
#pragma unroll
                for (int j = 0; j < 8; ++j) e[j] = (sc + j < o.col_lim) ? (uint32_t)q[j] : 0u;
                v.x = e[0] | (e[1] << 16);
                v.y = e[2] | (e[3] << 16);
                v.z = e[4] | (e[5] << 16);
                v.w = e[6] | (e[7] << 16);
            }
        }
        fr.q[i] = v;
    }
}

__device__ __forceinline__ void stash_kc(bf16_t (*S)[LDH], int tid, const Frag& fr) {
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int f = tid + 256 * i;
        *reinterpret_cast<uint4*>(&S[f >> 2][(f & 3) << 3]) = fr.q[i];
    }
}

// mn-contiguous storage (k, mn): each thread takes a pair of adjacent mn and 8 consecutive k
// (eight 4-byte loads, each wavefront reading 256 contiguous bytes), then repacks to two k-runs.
__device__ __forceinline__ void fetch_mc(const OperandViewH& o, int mn0, int k0, int tid, Frag& fr) {
    const int m2 = tid & 63, kg = tid >> 6;
    const int sc = mn0 + 2 * m2;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        const int sr = k0 + 8 * kg + j;
        uint32_t w = 0u;
        if (sr < o.row_lim) {
            const bf16_t* q = o.p + (long)sr * o.ld + sc;
            if (sc + 1 < o.col_lim) {
                w = *reinterpret_cast<const uint32_t*>(q);
            } else if (sc < o.col_lim) {
                w = (uint32_t)q[0];
            }
        }
        fr.w[j] = w;
    }
}

__device__ __forceinline__ void stash_mc(bf16_t (*S)[LDH], int tid, const Frag& fr) {
    const int m2 = tid & 63, kg = tid >> 6;
    uint4 lo, hi;
    lo.x = (fr.w[0] & 0xffffu) | (fr.w[1] << 16);
    lo.y = (fr.w[2] & 0xffffu) | (fr.w[3] << 16);
    lo.z = (fr.w[4] & 0xffffu) | (fr.w[5] << 16);
    lo.w = (fr.w[6] & 0xffffu) | (fr.w[7] << 16);
    hi.x = (fr.w[0] >> 16) | (fr.w[1] & 0xffff0000u);
    hi.y = (fr.w[2] >> 16) | (fr.w[3] & 0xffff0000u);
    hi.z = (fr.w[4] >> 16) | (fr.w[5] & 0xffff0000u);
    hi.w = (fr.w[6] >> 16) | (fr.w[7] & 0xffff0000u);
    *reinterpret_cast<uint4*>(&S[2 * m2][8 * kg]) = lo;
    *reinterpret_cast<uint4*>(&S[2 * m2 + 1][8 * kg]) = hi;
}

template <bool TA, bool TB>
__global__ __launch_bounds__(256) void gemm_bf16_kernel(GemmBf16 g, int tiles_m, int tiles_n, int avec, int bvec) {
    __shared__ __attribute__((aligned(16))) bf16_t As[2][BM][LDH];
    __shared__ __attribute__((aligned(16))) bf16_t Bs[2][BN][LDH];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;

    // XCD-aware tile order (see gemm_f32.hip)
    const int nt = tiles_m * tiles_n;
    const int bid = blockIdx.x;
    const int q8 = nt >> 3, r8 = nt & 7;
    const int xcd = bid & 7;
    const int pid = xcd * q8 + (xcd < r8 ? xcd : r8) + (bid >> 3);
    const int group = 8 * tiles_n;
    const int gid = pid / group;
    const int first_m = gid * 8;
    const int gsz = (tiles_m - first_m) < 8 ? (tiles_m - first_m) : 8;
    const int pid_m = first_m + (pid % group) % gsz;
    const int pid_n = (pid % group) / gsz;
    const int m0 = pid_m * BM, n0 = pid_n * BN;

    const int z = blockIdx.y;
    int kb = 0, ke = g.K;
    if (g.splits > 1) {
        kb = z * g.kchunk;
        ke = kb + g.kchunk < g.K ? kb + g.kchunk : g.K;
    }

    OperandViewH oa, ob;
    oa.p = g.A; oa.ld = g.lda; oa.vec = avec;
    if (TA) { oa.row_lim = ke; oa.col_lim = g.M; } else { oa.row_lim = g.M; oa.col_lim = ke; }
    const int wrap = g.a_kwrap;
    if (wrap > 0) { if (TA) oa.row_lim = g.a_klim; else oa.col_lim = g.a_klim; }
    ob.p = g.B; ob.ld = g.ldb; ob.vec = bvec;
    if (TB) { ob.row_lim = g.N; ob.col_lim = ke; } else { ob.row_lim = ke; ob.col_lim = g.N; }

    f32x16 acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    const int wm = (wave >> 1) * 64, wn = (wave & 1) * 64;
    const int lrow = lane & 31, lk = lane >> 5;

    const int nk = ke > kb ? (ke - kb + BK - 1) / BK : 0;
    Frag fa, fb;
    if (nk > 0) {
        const int ka = (wrap > 0 && kb >= wrap) ? kb - wrap : kb;
        if (TA) fetch_mc(oa, m0, ka, tid, fa); else fetch_kc(oa, m0, ka, tid, fa);
        if (TB) fetch_kc(ob, n0, kb, tid, fb); else fetch_mc(ob, n0, kb, tid, fb);
        if (TA) stash_mc(As[0], tid, fa); else stash_kc(As[0], tid, fa);
        if (TB) stash_kc(Bs[0], tid, fb); else stash_mc(Bs[0], tid, fb);
    }
    __syncthreads();
    for (int kt = 0; kt < nk; ++kt) {
        const int cur = kt & 1;
        if (kt + 1 < nk) {
            const int k0 = kb + (kt + 1) * BK;
            const int ka = (wrap > 0 && k0 >= wrap) ? k0 - wrap : k0;
            if (TA) fetch_mc(oa, m0, ka, tid, fa); else fetch_kc(oa, m0, ka, tid, fa);
            if (TB) fetch_kc(ob, n0, k0, tid, fb); else fetch_mc(ob, n0, k0, tid, fb);
        }
#pragma unroll
        for (int ks = 0; ks < BK; ks += 16) {
            bf16x8 a[2], b[2];
#pragma unroll
            for (int i = 0; i < 2; ++i)
                a[i] = *reinterpret_cast<const bf16x8*>(&As[cur][wm + i * 32 + lrow][ks + lk * 8]);
#pragma unroll
            for (int j = 0; j < 2; ++j)
                b[j] = *reinterpret_cast<const bf16x8*>(&Bs[cur][wn + j * 32 + lrow][ks + lk * 8]);
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int j = 0; j < 2; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[j], acc[i][j], 0, 0, 0);
        }
        if (kt + 1 < nk) {
            if (TA) stash_mc(As[cur ^ 1], tid, fa); else stash_kc(As[cur ^ 1], tid, fa);
            if (TB) stash_kc(Bs[cur ^ 1], tid, fb); else stash_mc(Bs[cur ^ 1], tid, fb);
        }
        __syncthreads();
    }

    float* C = g.C + (long)z * g.split_stride;
#pragma unroll
    for (int i = 0; i < 2; ++i) {
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const int col = n0 + wn + j * 32 + lrow;
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int row = m0 + wm + i * 32 + 8 * (v >> 2) + 4 * lk + (v & 3);
                if (row < g.M && col < g.N) C[(long)row * g.ldc + col] = acc[i][j][v];
            }
        }
    }
}

// ---- large "NT" products (both operands k-contiguous: A is M x K, B is N x K) ---------------------------------
// Same 128 x 128 tile and wavefront layout as above, but a K step of 64 (16 MFMAs per wavefront between two
// barriers), without guards (M, N multiples of 128, K of 128, 16-byte aligned rows; a_kwrap a multiple of 64 with
// a_klim == a_kwrap) and with TWO K steps (128 reduction indices) of operands in flight in registers: a K step is far
// shorter than the memory latency, and two workgroups per compute unit do not hide it.  The loop body has no early
// exit (K % 128 == 0).
constexpr int BKD = 64;
constexpr int LDD = BKD + 8;   // LDS row stride in halfwords (144 bytes)
__device__ __forceinline__ void multiply_tile(const bf16_t (*Asc)[LDD], const bf16_t (*Bsc)[LDD], f32x16 (&acc)[2][2],
                                              int wm, int wn, int lrow, int lk) {
#pragma unroll
    for (int ks = 0; ks < BKD; ks += 16) {
        bf16x8 a[2], b[2];
#pragma unroll
        for (int i = 0; i < 2; ++i) a[i] = *reinterpret_cast<const bf16x8*>(&Asc[wm + i * 32 + lrow][ks + lk * 8]);
#pragma unroll
        for (int j = 0; j < 2; ++j) b[j] = *reinterpret_cast<const bf16x8*>(&Bsc[wn + j * 32 + lrow][ks + lk * 8]);
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int j = 0; j < 2; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[j], acc[i][j], 0, 0, 0);
    }
}

// WHIP: the epilogue applies the Whip loss and its derivative (Eq. 4; the loss step of Alg. 1) to the accumulators instead of
// (or beside) writing them: per-workgroup partial sums of exp(-|y|) go to g.whip_partials[workgroup], and
// dY = -scale sgn(y) exp(-|y|) is written TRANSPOSED in bf16 (g.whip_dyt: N x M, token-contiguous), staged through
// the operand buffers in LDS so that every row of 128 tokens leaves as one 256-byte run.
template <bool WHIP>
__global__ __launch_bounds__(256) void gemm_bf16_nt_deep_kernel(GemmBf16 g, int tiles_m, int tiles_n) {
    __shared__ __attribute__((aligned(16))) bf16_t smem[2 * BM * LDD + 2 * BN * LDD];
    bf16_t (*As)[BM][LDD] = reinterpret_cast<bf16_t (*)[BM][LDD]>(smem);
    bf16_t (*Bs)[BN][LDD] = reinterpret_cast<bf16_t (*)[BN][LDD]>(smem + 2 * BM * LDD);

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;

    // XCD-aware tile order (see gemm_f32.hip)
    const int nt = tiles_m * tiles_n;
    const int bid = blockIdx.x;
    const int q8 = nt >> 3, r8 = nt & 7;
    const int xcd = bid & 7;
    const int pid = xcd * q8 + (xcd < r8 ? xcd : r8) + (bid >> 3);
    const int group = 8 * tiles_n;
    const int gid = pid / group;
    const int first_m = gid * 8;
    const int gsz = (tiles_m - first_m) < 8 ? (tiles_m - first_m) : 8;
    const int pid_m = first_m + (pid % group) % gsz;
    const int pid_n = (pid % group) / gsz;
    const int m0 = pid_m * BM, n0 = pid_n * BN;

    const int wrap = g.a_kwrap;

    f32x16 acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    const int wm = (wave >> 1) * 64, wn = (wave & 1) * 64;
    const int lrow = lane & 31, lk = lane >> 5;

    // thread t moves the 16-byte piece (row t / 8 + 32 i, k-offset 8 (t % 8)) of each operand tile, i = 0 .. 3
    const int prow = tid >> 3, pk = (tid & 7) << 3;
    const bf16_t* pa = g.A + (long)(m0 + prow) * g.lda + pk;
    const bf16_t* pb = g.B + (long)(n0 + prow) * g.ldb + pk;
    const long sa = 32 * g.lda, sb = 32 * g.ldb;

    const int nk = g.K / BKD;
    struct Stage { uint4 a0, a1, a2, a3, b0, b1, b2, b3; };
    Stage st0, st1;

#define DQ_FETCH(kt, st)                                                                           \
    if ((kt) < nk) {                                                                               \
        const int k0_ = (kt) * BKD;                                                                \
        const int ka_ = (wrap > 0 && k0_ >= wrap) ? k0_ - wrap : k0_;                              \
        st.a0 = *reinterpret_cast<const uint4*>(pa + ka_);                                         \
        st.a1 = *reinterpret_cast<const uint4*>(pa + sa + ka_);                                    \
        st.a2 = *reinterpret_cast<const uint4*>(pa + 2 * sa + ka_);                                \
        st.a3 = *reinterpret_cast<const uint4*>(pa + 3 * sa + ka_);                                \
        st.b0 = *reinterpret_cast<const uint4*>(pb + k0_);                                         \
        st.b1 = *reinterpret_cast<const uint4*>(pb + sb + k0_);                                    \
        st.b2 = *reinterpret_cast<const uint4*>(pb + 2 * sb + k0_);                                \
        st.b3 = *reinterpret_cast<const uint4*>(pb + 3 * sb + k0_);                                \
    }
#define DQ_STASH(buf, st)                                                                          \
    {                                                                                              \
        *reinterpret_cast<uint4*>(&As[buf][prow][pk]) = st.a0;                                     \
        *reinterpret_cast<uint4*>(&As[buf][prow + 32][pk]) = st.a1;                                \
        *reinterpret_cast<uint4*>(&As[buf][prow + 64][pk]) = st.a2;                                \
        *reinterpret_cast<uint4*>(&As[buf][prow + 96][pk]) = st.a3;                                \
        *reinterpret_cast<uint4*>(&Bs[buf][prow][pk]) = st.b0;                                     \
        *reinterpret_cast<uint4*>(&Bs[buf][prow + 32][pk]) = st.b1;                                \
        *reinterpret_cast<uint4*>(&Bs[buf][prow + 64][pk]) = st.b2;                                \
        *reinterpret_cast<uint4*>(&Bs[buf][prow + 96][pk]) = st.b3;                                \
    }
#define DQ_MULTIPLY(cur) multiply_tile(As[cur], Bs[cur], acc, wm, wn, lrow, lk);
    // tile kt is in LDS buffer `buf`, tile kt+1 in st_next; tile kt+2 is requested into the registers that held tile kt
#define DQ_STEP(kt, buf, st_next, st_free)                                                         \
    {                                                                                              \
        DQ_FETCH((kt) + 2, st_free)                                                                \
        DQ_MULTIPLY(buf)                                                                           \
        if ((kt) + 1 < nk) { DQ_STASH(1 - (buf), st_next) }                                        \
        __syncthreads();                                                                           \
    }
    st0.a0 = st0.a1 = st0.a2 = st0.a3 = st0.b0 = st0.b1 = st0.b2 = st0.b3 = make_uint4(0u, 0u, 0u, 0u);
    st1 = st0;
    DQ_FETCH(0, st0)
    DQ_FETCH(1, st1)
    DQ_STASH(0, st0)
    __syncthreads();
    for (int kt = 0; kt < nk; kt += 2) {
        DQ_STEP(kt, 0, st1, st0)
        DQ_STEP(kt + 1, 1, st0, st1)
    }
#undef DQ_STEP
#undef DQ_MULTIPLY
#undef DQ_STASH
#undef DQ_FETCH

    float* C = g.C;
    if (!WHIP || C != nullptr) {
#pragma unroll
        for (int i = 0; i < 2; ++i) {
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                const int col = n0 + wn + j * 32 + lrow;
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int row = m0 + wm + i * 32 + 8 * (v >> 2) + 4 * lk + (v & 3);
                    C[(long)row * g.ldc + col] = acc[i][j][v];
                }
            }
        }
    }
    if constexpr (WHIP) {
        typedef float f32x2 __attribute__((ext_vector_type(2)));
        typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
        constexpr int SLD = BM + 8;          // halfwords per staged row (272 bytes)
        static_assert(BN * SLD <= 2 * BM * LDD + 2 * BN * LDD, "the staged tile must fit the operand buffers");
        bf16_t* stage = smem;                // [BN][SLD]; the K loop ended with a barrier: the buffers are free
        const float scale = g.whip_scale;
        float lsum = 0.f;
#pragma unroll
        for (int i = 0; i < 2; ++i) {
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                const int c = wn + j * 32 + lrow;
#pragma unroll
                for (int q4 = 0; q4 < 4; ++q4) {
                    const int r0 = wm + i * 32 + 8 * q4 + 4 * lk;
                    float d[4];
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        const float y = acc[i][j][4 * q4 + q];
                        const float ex = __expf(-fabsf(y));
                        lsum += ex;
                        const float sg = (y > 0.f) ? -scale : ((y < 0.f) ? scale : 0.f);
                        d[q] = sg * ex;
                    }
                    const f32x2 d01 = {d[0], d[1]}, d23 = {d[2], d[3]};
                    const bf16x2 b01 = __builtin_convertvector(d01, bf16x2), b23 = __builtin_convertvector(d23, bf16x2);
                    *reinterpret_cast<uint2*>(stage + c * SLD + r0) =
                        make_uint2(__builtin_bit_cast(uint32_t, b01), __builtin_bit_cast(uint32_t, b23));
                }
            }
        }
        __syncthreads();
#pragma unroll
        for (int pass = 0; pass < BN / 16; ++pass) {
            const int row = pass * 16 + (tid >> 4), piece = (tid & 15) * 8;
            const uint4 v = *reinterpret_cast<const uint4*>(stage + row * SLD + piece);
            *reinterpret_cast<uint4*>(g.whip_dyt + (long)(n0 + row) * g.whip_ldt + m0 + piece) = v;
        }
        __shared__ float wsum[4];
#pragma unroll
        for (int o = 32; o >= 1; o >>= 1) lsum += __shfl_xor(lsum, o);
        if (lane == 0) wsum[wave] = lsum;
        __syncthreads();
        if (tid == 0)
            g.whip_partials[bid] = (double)wsum[0] + (double)wsum[1] + (double)wsum[2] + (double)wsum[3];
    }
}


// ---- the same products on 256 x 256 x 64 tiles ------------------------------------------------------------------
// One workgroup of 4 wavefronts per compute unit, each wavefront a 128 x 128 block (4 x 4 MFMA tiles: 256 accumulator
// registers, half as many LDS reads per MFMA as the 64 x 64 blocks above and half the operand traffic out of L2 per
// flop, which is what bounds the 128 x 128 kernel).  With one wavefront per SIMD nothing else hides latencies, so the
// K step is written out as 64 "slots", one MFMA each, and every memory operation is given its slot by hand (a
// scheduling barrier after each slot keeps the compiler from regrouping them; without the barriers the same code runs
// 15 % slower):
//   * the fragments of reduction sub-step s + 1 are read from LDS in the first 8 slots of sub-step s (the last
//     sub-step reads the first fragments of the NEXT tile from the other LDS buffer);
//   * the 16 staged 16-byte pieces per thread of the next tile go to the other LDS buffer in slots 0, 3, .., 45, and
//     each staging register is reloaded with its piece of the tile two steps further in slot 4 p + 3: two K steps of
//     global loads are always in flight (about 3 us at the rate reached);
//   * one barrier per K step, before its last sub-step: by then every wavefront has read the last fragments of the
//     current buffer and written its pieces of the next one.
// Shapes: M, N multiples of 256, K of 128, the other conditions of the kernel above.
constexpr int TM = 256, TN = 256, TK = 64;
constexpr int TLD = TK + 8;                         // LDS row stride in halfwords (144 bytes)
constexpr int kBigAbuf = TM * TLD, kBigBbase = 2 * TM * TLD, kBigBbuf = TN * TLD;   // halfword offsets in LDS

struct BigAcc { f32x16 t[4][4]; };
// Register sets with named members and compile-time selectors: arrays indexed inside loops that are only unrolled
// later in the compilation end up in scratch memory.
struct BigFrags { bf16x8 a0, a1, a2, a3, b0, b1, b2, b3; };
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));   // a native vector: copies are typed loads / stores
struct BigStage { u32x4 r0, r1, r2, r3, r4, r5, r6, r7, r8, r9, r10, r11, r12, r13, r14, r15; };   // pieces 0..7 of the A tile, 8..15 of the B tile
template <int I, class F> __device__ __forceinline__ auto& frag_a(F& f) {
    if constexpr (I == 0) return f.a0; else if constexpr (I == 1) return f.a1; else if constexpr (I == 2) return f.a2; else return f.a3;
}
template <int I, class F> __device__ __forceinline__ auto& frag_b(F& f) {
    if constexpr (I == 0) return f.b0; else if constexpr (I == 1) return f.b1; else if constexpr (I == 2) return f.b2; else return f.b3;
}
template <int P> __device__ __forceinline__ u32x4& piece(BigStage& s) {
    if constexpr (P == 0) return s.r0; else if constexpr (P == 1) return s.r1; else if constexpr (P == 2) return s.r2;
    else if constexpr (P == 3) return s.r3; else if constexpr (P == 4) return s.r4; else if constexpr (P == 5) return s.r5;
    else if constexpr (P == 6) return s.r6; else if constexpr (P == 7) return s.r7; else if constexpr (P == 8) return s.r8;
    else if constexpr (P == 9) return s.r9; else if constexpr (P == 10) return s.r10; else if constexpr (P == 11) return s.r11;
    else if constexpr (P == 12) return s.r12; else if constexpr (P == 13) return s.r13; else if constexpr (P == 14) return s.r14;
    else return s.r15;
}
struct BigAddr {
    const bf16_t* pa; const bf16_t* pb;             // this thread's first piece of the tile being fetched
    long sa, sb;                                    // 32 rows further
    int aoff, boff;                                 // halfword offsets of this lane's fragment rows in an operand buffer
    int sto;                                        // halfword offset of this thread's first piece in an operand buffer
};

template <int KS, int BUF, int Q>
__device__ __forceinline__ void big_slot(BigAcc& acc, const BigFrags& cur, BigFrags& nxt, BigStage& st, const BigAddr& ad,
                                         bf16_t* smem) {
    constexpr int i = Q >> 2, j = (i & 1) ? 3 - (Q & 3) : (Q & 3);
    acc.t[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_a<i>(cur), frag_b<j>(cur), acc.t[i][j], 0, 0, 0);
    constexpr int RB = (KS == 3) ? 1 - BUF : BUF;        // buffer and k offset of the fragments read now
    constexpr int RK = (KS == 3) ? 0 : (KS + 1) * 16;
    if constexpr (Q < 4)
        frag_a<Q>(nxt) = *reinterpret_cast<const bf16x8*>(smem + RB * kBigAbuf + ad.aoff + Q * 32 * TLD + RK);
    else if constexpr (Q < 8)
        frag_b<Q - 4>(nxt) = *reinterpret_cast<const bf16x8*>(smem + kBigBbase + RB * kBigBbuf + ad.boff + (Q - 4) * 32 * TLD + RK);
    constexpr int S = KS * 16 + Q;                       // slot number inside the K step
    if constexpr (S % 3 == 0 && S / 3 < 16) {
        constexpr int P = S / 3;
        if constexpr (P < 8)
            *reinterpret_cast<u32x4*>(smem + (1 - BUF) * kBigAbuf + ad.sto + P * 32 * TLD) = piece<P>(st);
        else
            *reinterpret_cast<u32x4*>(smem + kBigBbase + (1 - BUF) * kBigBbuf + ad.sto + (P - 8) * 32 * TLD) = piece<P>(st);
    }
    if constexpr (S % 4 == 3) {
        constexpr int P = S / 4;
        if constexpr (P < 8) piece<P>(st) = *reinterpret_cast<const u32x4*>(ad.pa + P * ad.sa);
        else piece<P>(st) = *reinterpret_cast<const u32x4*>(ad.pb + (P - 8) * ad.sb);
    }
    __builtin_amdgcn_sched_barrier(0);
}

// all 16 pieces of the tile at ad.pa / ad.pb into st
template <int... P>
__device__ __forceinline__ void big_fetch(BigStage& st, const BigAddr& ad, std::integer_sequence<int, P...>) {
    ((piece<P>(st) = *reinterpret_cast<const u32x4*>(P < 8 ? ad.pa + P * ad.sa : ad.pb + (P - 8) * ad.sb)), ...);
}
// st into LDS buffer 0
template <int... P>
__device__ __forceinline__ void big_stash0(BigStage& st, const BigAddr& ad, bf16_t* smem, std::integer_sequence<int, P...>) {
    ((*reinterpret_cast<u32x4*>(smem + (P < 8 ? 0 : kBigBbase) + ad.sto + (P & 7) * 32 * TLD) = piece<P>(st)), ...);
}
// the first fragments of the tile in LDS buffer 0
template <int... Q>
__device__ __forceinline__ void big_first_frags(BigFrags& f, const BigAddr& ad, const bf16_t* smem, std::integer_sequence<int, Q...>) {
    ((frag_a<Q>(f) = *reinterpret_cast<const bf16x8*>(smem + ad.aoff + Q * 32 * TLD)), ...);
    ((frag_b<Q>(f) = *reinterpret_cast<const bf16x8*>(smem + kBigBbase + ad.boff + Q * 32 * TLD)), ...);
}

template <int KS, int BUF, int... Q>
__device__ __forceinline__ void big_substep(BigAcc& acc, const BigFrags& cur, BigFrags& nxt, BigStage& st,
                                            const BigAddr& ad, bf16_t* smem, std::integer_sequence<int, Q...>) {
    (big_slot<KS, BUF, Q>(acc, cur, nxt, st, ad, smem), ...);
}

// One K step on the tile in LDS buffer BUF (its first fragments in f0): stashes `st` (the next tile) into the other
// buffer, reloads `st` from ad.pa / ad.pb, and leaves the first fragments of the next tile in f0.
template <int BUF>
__device__ __forceinline__ void big_kstep(BigAcc& acc, BigFrags& f0, BigFrags& f1, BigStage& st, const BigAddr& ad,
                                          bf16_t* smem) {
    using Seq = std::make_integer_sequence<int, 16>;
    big_substep<0, BUF>(acc, f0, f1, st, ad, smem, Seq{});
    big_substep<1, BUF>(acc, f1, f0, st, ad, smem, Seq{});
    big_substep<2, BUF>(acc, f0, f1, st, ad, smem, Seq{});
    __syncthreads();
    big_substep<3, BUF>(acc, f1, f0, st, ad, smem, Seq{});
}

// X3: the operands are three bf16 planes each (x = x1 + x2 + x3 to 24 mantissa bits, plane p at + p * a_plane / b_plane
// elements) and the reduction runs over six segments of K indices, one per pair of planes whose product is not below
// fp32 rounding -- (3,1) (1,3) (2,2) (2,1) (1,2) (1,1), small terms first -- into the same fp32 accumulators: an fp32
// product on the bf16 matrix cores (each bf16 x bf16 product is exact in fp32; the three pairs left out are below
// 2^-26 of |a| |b|).  Epilogue C = alpha * acc + beta * C.  With b_strict_lower the segments start at the tile's
// first column (B^T vanishes on and above the diagonal) and tiles are taken column block by column block, the
// longest reductions first.
template <bool WHIP, bool X3 = false>
__global__ __launch_bounds__(256, 1) void gemm_bf16_nt_big_kernel(GemmBf16 g, int tiles_m, int tiles_n) {
    __shared__ __attribute__((aligned(16))) bf16_t smem[2 * TM * TLD + 2 * TN * TLD];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;

    // XCD-aware tile order (see gemm_f32.hip): the 32 workgroups resident on an XCD form an 8 x 4 block of tiles
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
    int zsplit = 0;
    if (X3 && g.b_strict_lower) {
        // column block by column block, the longest reductions first; with split-K the parts of a tile side by side
        const int per_col = tiles_m * (g.splits > 1 ? g.splits : 1);
        pid_n = bid / per_col;
        zsplit = (bid % per_col) / tiles_m;
        pid_m = bid % tiles_m;
    }
    const int m0 = pid_m * TM, n0 = pid_n * TN;

    const int wm = (wave >> 1) * 128, wn = (wave & 1) * 128;
    const int lrow = lane & 31, lk = lane >> 5;
    // thread t moves the 16-byte piece (row t / 8 + 32 i, k-offset 8 (t % 8)) of each operand tile, i = 0 .. 7
    const int prow = tid >> 3, pk = (tid & 7) << 3;
    const bf16_t* pa = g.A + (long)(m0 + prow) * g.lda + pk;
    const bf16_t* pb = g.B + (long)(n0 + prow) * g.ldb + pk;
    const int wrap = g.a_kwrap;
    int kbeg = (X3 && g.b_strict_lower) ? n0 : 0;
    int kend = g.K;
    if (X3 && g.splits > 1) {
        // split-K (with b_strict_lower only): part z of the tile's reduction range, in whole K steps, into C + z * split_stride
        const int part = (((kend - kbeg) / TK + g.splits - 1) / g.splits) * TK;
        kbeg += zsplit * part;
        kend = kbeg + part < kend ? kbeg + part : kend;
    }
    const int nk = X3 ? 6 * ((kend - kbeg) / TK) : g.K / TK;           // even, >= 2

    BigAddr ad;
    ad.sa = 32 * g.lda; ad.sb = 32 * g.ldb;
    ad.aoff = (wm + lrow) * TLD + lk * 8; ad.boff = (wn + lrow) * TLD + lk * 8;
    ad.sto = prow * TLD + pk;
    // tile t (clamped to the last one: past the end a valid tile is fetched again and never used)
    // X3: the calls below ask for tiles 0, 1, 2, ... in order, so the segment and the index inside it are carried along
    int seg = 0, kk = kbeg;
    long offa = 2 * g.a_plane, offb = 0;
    auto point_at = [&](int t) {
        if constexpr (X3) {
            ad.pa = pa + offa + kk;
            ad.pb = pb + offb + kk;
            kk += TK;
            if (kk == kend) {
                if (seg < 5) {
                    kk = kbeg;
                    ++seg;
                    offa = ((0x052 >> (2 * seg)) & 3) * g.a_plane;     // planes 3 1 2 2 1 1 of A ...
                    offb = ((0x118 >> (2 * seg)) & 3) * g.b_plane;     // ... against planes 1 3 2 1 2 1 of B
                } else {
                    kk -= TK;
                }
            }
        } else {
            const int tc = t < nk ? t : nk - 1;
            const int k0 = tc * TK;
            ad.pa = pa + ((wrap > 0 && k0 >= wrap) ? k0 - wrap : k0);
            ad.pb = pb + k0;
        }
    };

    BigAcc acc;
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc.t[i][j][v] = 0.f;

    BigStage s0, s1;
    BigFrags f0, f1;
    using Seq16 = std::make_integer_sequence<int, 16>;
    point_at(0);
    big_fetch(s0, ad, Seq16{});
    point_at(1);
    big_fetch(s1, ad, Seq16{});
    big_stash0(s0, ad, smem, Seq16{});
    point_at(2);
    big_fetch(s0, ad, Seq16{});
    __syncthreads();
    big_first_frags(f0, ad, smem, std::make_integer_sequence<int, 4>{});
    // at the top of a trip: tile kt in LDS buffer 0 with its first fragments in f0, tile kt + 1 in s1, tile kt + 2 in s0
    for (int kt = 0; kt < nk; kt += 2) {
        point_at(kt + 3);
        big_kstep<0>(acc, f0, f1, s1, ad, smem);
        point_at(kt + 4);
        big_kstep<1>(acc, f0, f1, s0, ad, smem);
    }

    float* C = g.C;
    float alpha = g.alpha;
    if constexpr (X3) {
        if (g.alpha_dev != nullptr) alpha *= *g.alpha_dev;
        C += (long)zsplit * g.split_stride;
    }
    if (!WHIP || C != nullptr) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int col = n0 + wn + j * 32 + lrow;
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int row = m0 + wm + i * 32 + 8 * (v >> 2) + 4 * lk + (v & 3);
                    if constexpr (X3) {
                        float r = alpha * acc.t[i][j][v];
                        if (g.beta != 0.f) r += g.beta * C[(long)row * g.ldc + col];
                        C[(long)row * g.ldc + col] = r;
                    } else {
                        C[(long)row * g.ldc + col] = acc.t[i][j][v];
                    }
                }
            }
        }
    }
    if constexpr (WHIP) {
        // as in the 128 x 128 kernel: dY leaves transposed, every row of 256 tokens as one 512-byte run
        typedef float f32x2 __attribute__((ext_vector_type(2)));
        typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
        constexpr int SLD = TM + 8;          // halfwords per staged row (528 bytes)
        static_assert(TN * SLD <= 2 * TM * TLD + 2 * TN * TLD, "the staged tile must fit the operand buffers");
        __syncthreads();                     // the last K step read fragments after its barrier
        bf16_t* stage = smem;                // [TN][SLD]
        const float scale = g.whip_scale;
        float lsum = 0.f;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int c = wn + j * 32 + lrow;
#pragma unroll
                for (int q4 = 0; q4 < 4; ++q4) {
                    const int r0 = wm + i * 32 + 8 * q4 + 4 * lk;
                    float d[4];
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        const float y = acc.t[i][j][4 * q4 + q];
                        const float ex = __expf(-fabsf(y));
                        lsum += ex;
                        const float sg = (y > 0.f) ? -scale : ((y < 0.f) ? scale : 0.f);
                        d[q] = sg * ex;
                    }
                    const f32x2 d01 = {d[0], d[1]}, d23 = {d[2], d[3]};
                    const bf16x2 b01 = __builtin_convertvector(d01, bf16x2), b23 = __builtin_convertvector(d23, bf16x2);
                    *reinterpret_cast<uint2*>(stage + c * SLD + r0) =
                        make_uint2(__builtin_bit_cast(uint32_t, b01), __builtin_bit_cast(uint32_t, b23));
                }
            }
        }
        __syncthreads();
#pragma unroll 4
        for (int pass = 0; pass < TN / 8; ++pass) {
            const int row = pass * 8 + (tid >> 5), piece = (tid & 31) * 8;
            const uint4 v = *reinterpret_cast<const uint4*>(stage + row * SLD + piece);
            *reinterpret_cast<uint4*>(g.whip_dyt + (long)(n0 + row) * g.whip_ldt + m0 + piece) = v;
        }
        __shared__ float wsum[4];
#pragma unroll
        for (int o = 32; o >= 1; o >>= 1) lsum += __shfl_xor(lsum, o);
        if (lane == 0) wsum[wave] = lsum;
        __syncthreads();
        if (tid == 0)
            g.whip_partials[bid] = (double)wsum[0] + (double)wsum[1] + (double)wsum[2] + (double)wsum[3];
    }
}

}  // namespace

// The 256 x 256 kernel needs enough tiles to give every compute unit one.
static bool gemm_bf16_big_fits(const GemmBf16& g) {
    return gemm_bf16_deep_fits(g) && g.M % TM == 0 && g.N % TN == 0 && (g.M / TM) * (g.N / TN) >= 192;
}

int gemm_bf16_whip_partials(const GemmBf16& g) {
    if (gemm_bf16_big_fits(g)) return (g.M / TM) * (g.N / TN);
    return (g.M / BM) * (g.N / BN);
}

bool gemm_bf16_deep_fits(const GemmBf16& g) {
    const int tiles_m = (g.M + BM - 1) / BM, tiles_n = (g.N + BN - 1) / BN;
    const bool avec = (reinterpret_cast<uintptr_t>(g.A) & 15) == 0 && (g.lda & 7) == 0;
    const bool bvec = (reinterpret_cast<uintptr_t>(g.B) & 15) == 0 && (g.ldb & 7) == 0;
    return !g.ta && g.tb && g.splits <= 1 && g.M % BM == 0 && g.N % BN == 0 && g.K % (2 * BKD) == 0 &&
           tiles_m * tiles_n >= 256 && avec && bvec && (g.a_kwrap == 0 || (g.a_kwrap % BKD == 0 && g.a_klim == g.a_kwrap));
}

bool gemm_bf16x3_fits(int M, int N, int K) { return M > 0 && N > 0 && K > 0 && M % TM == 0 && N % TN == 0 && K % TK == 0; }

hipError_t launch_gemm_bf16x3(const GemmBf16& g, hipStream_t s) {
    // split-K: only for the triangular product, every part at least two K steps (the shortest range is one tile width)
    const bool split_ok = g.splits <= 1 || (g.b_strict_lower && g.splits <= TN / (2 * TK) && g.split_stride > 0);
    if (!gemm_bf16x3_fits(g.M, g.N, g.K) || g.ta || !g.tb || !split_ok || g.a_kwrap != 0 || g.whip_dyt != nullptr ||
        (reinterpret_cast<uintptr_t>(g.A) & 15) || (reinterpret_cast<uintptr_t>(g.B) & 15) || (g.lda & 7) || (g.ldb & 7) ||
        (g.a_plane & 7) || (g.b_plane & 7) || g.C == nullptr || (g.b_strict_lower && g.K != g.N))
        return hipErrorInvalidValue;
    const int parts = g.splits > 1 ? g.splits : 1;
    hipLaunchKernelGGL((gemm_bf16_nt_big_kernel<false, true>), dim3((g.M / TM) * (g.N / TN) * parts), dim3(256), 0, s, g,
                       g.M / TM, g.N / TN);
    return hipGetLastError();
}

hipError_t launch_gemm_bf16(const GemmBf16& g, hipStream_t s) {
    if (g.M <= 0 || g.N <= 0) return hipSuccess;
    const int tiles_m = (g.M + BM - 1) / BM, tiles_n = (g.N + BN - 1) / BN;
    const int avec = ((reinterpret_cast<uintptr_t>(g.A) & 15) == 0 && (g.lda & 7) == 0) ? 1 : 0;
    const int bvec = ((reinterpret_cast<uintptr_t>(g.B) & 15) == 0 && (g.ldb & 7) == 0) ? 1 : 0;
    // big NT products without split-K and with round sizes: the unguarded kernel with the deep prefetch
    const bool fits = gemm_bf16_deep_fits(g);
    const bool big = gemm_bf16_big_fits(g);
    if (g.whip_dyt != nullptr) {   // the fused epilogue exists in the unguarded kernel only: the caller checks first
        if (!fits || g.whip_partials == nullptr || (g.whip_ldt & 7) != 0 || g.whip_ldt < g.M ||
            (reinterpret_cast<uintptr_t>(g.whip_dyt) & 15) != 0)
            return hipErrorInvalidValue;
        if (big)
            hipLaunchKernelGGL((gemm_bf16_nt_big_kernel<true>), dim3((g.M / TM) * (g.N / TN)), dim3(256), 0, s, g,
                               g.M / TM, g.N / TN);
        else
            hipLaunchKernelGGL((gemm_bf16_nt_deep_kernel<true>), dim3(tiles_m * tiles_n), dim3(256), 0, s, g, tiles_m,
                               tiles_n);
        return hipGetLastError();
    }
    if (big) {
        hipLaunchKernelGGL((gemm_bf16_nt_big_kernel<false>), dim3((g.M / TM) * (g.N / TN)), dim3(256), 0, s, g, g.M / TM,
                           g.N / TN);
        return hipGetLastError();
    }
    if (fits) {
        hipLaunchKernelGGL((gemm_bf16_nt_deep_kernel<false>), dim3(tiles_m * tiles_n), dim3(256), 0, s, g, tiles_m,
                           tiles_n);
        return hipGetLastError();
    }
    dim3 grid(tiles_m * tiles_n, g.splits > 1 ? g.splits : 1, 1);
    dim3 block(256, 1, 1);
    if (g.ta && g.tb)
        hipLaunchKernelGGL((gemm_bf16_kernel<true, true>), grid, block, 0, s, g, tiles_m, tiles_n, avec, bvec);
    else if (g.ta)
        hipLaunchKernelGGL((gemm_bf16_kernel<true, false>), grid, block, 0, s, g, tiles_m, tiles_n, avec, bvec);
    else if (g.tb)
        hipLaunchKernelGGL((gemm_bf16_kernel<false, true>), grid, block, 0, s, g, tiles_m, tiles_n, avec, bvec);
    else
        hipLaunchKernelGGL((gemm_bf16_kernel<false, false>), grid, block, 0, s, g, tiles_m, tiles_n, avec, bvec);
    return hipGetLastError();
}

}  // namespace dq
