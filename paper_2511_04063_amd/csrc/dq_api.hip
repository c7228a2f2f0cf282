// C ABI of libdartqr.so: argument checking, workspace carving and the sequencing of the kernels of one
// QR-Orth step (the loop body of Alg. 1) on the caller's HIP stream.  No device memory is allocated here.
#include <math.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <mutex>
#include <new>
#include <vector>

#include "dq_internal.h"

namespace dq {

// ---------------------------------------------------------------- profiling
struct Profiler {
    unsigned mask = 0;
    struct Rec { int klass; double flops, bytes; };
    std::vector<hipEvent_t> ev;   // two per record
    std::vector<Rec> recs;
    bool failed = false;
    int acquire(int klass, double flops, double bytes) {
        const size_t slot = recs.size();
        if (slot >= 65536) return -1;
        while (ev.size() < 2 * (slot + 1)) {
            hipEvent_t e;
            if (hipEventCreate(&e) != hipSuccess) { failed = true; return -1; }
            ev.push_back(e);
        }
        recs.push_back({klass, flops, bytes});
        return (int)slot;
    }
};

LaunchScope::LaunchScope(Profiler* p, hipStream_t s, int k, double flops, double bytes)
    : prof(p), stream(s), klass(k), slot(-1) {
    if (prof != nullptr && ((prof->mask >> k) & 1u)) {
        slot = prof->acquire(k, flops, bytes);
        if (slot >= 0 && hipEventRecord(prof->ev[2 * slot], stream) != hipSuccess) prof->failed = true;
    }
}
LaunchScope::~LaunchScope() {
    if (slot >= 0 && hipEventRecord(prof->ev[2 * slot + 1], stream) != hipSuccess) prof->failed = true;
}

}  // namespace dq

using namespace dq;

// ---------------------------------------------------------------- memory of the entry point that allocates nothing
// Device memory that dq_whip_loss_grad_noalloc uses in place of a caller's workspace: a status word (first 256
// bytes) and the per-workgroup partial sums of the loss.  Every GPU the library runs on holds its own copy of the
// array for the life of the process.  In host code the array's name is only a handle for hipGetSymbolAddress: the
// address kernels and fills are given is the one looked up below, once per device.
constexpr int kNoallocPartials = DQ_NOALLOC_MAX_BATCH;     // at least one partial per problem
constexpr size_t kNoallocBytes = 256 + (size_t)kNoallocPartials * sizeof(double);
static __device__ __align__(256) unsigned char scratch[kNoallocBytes];

namespace {
constexpr int kNoallocMaxDevices = 64;
std::mutex g_noalloc_mutex;
void* g_noalloc_ptr[kNoallocMaxDevices] = {};

// The device address of `scratch` on the current device (looked up on the first call on that device).
hipError_t noalloc_scratch(void** out) {
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kNoallocMaxDevices) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(g_noalloc_mutex);
    if (g_noalloc_ptr[dev] == nullptr) {
        void* p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (p == nullptr) return hipErrorInvalidSymbol;
        g_noalloc_ptr[dev] = p;
    }
    *out = g_noalloc_ptr[dev];
    return hipSuccess;
}
}  // namespace

struct dq_ctx {
    hipStream_t stream = nullptr;    // the caller's stream: every call starts and ends here
    hipStream_t stream2 = nullptr;   // internal: trailing updates of the QR run here while the next panel is factored
    hipStream_t stream3 = nullptr;   // internal: the orthogonal factor is accumulated here, also behind the panels
    std::vector<hipEvent_t> sync_ev; // 2 per panel: look-ahead part done (even), trailing part done (odd); + 1 join
    hipStream_t copy_stream = nullptr;   // internal, created on first use: host-to-device copies of the next mini-batch
    hipEvent_t batch_ready[2] = {nullptr, nullptr};   // staging slot holds its batch (recorded on copy_stream)
    hipEvent_t batch_done[2] = {nullptr, nullptr};    // the step that read the slot has run (recorded on stream)
    int device = 0;
    int chol_min_m = 64;             // full-width panels at least this tall take the many-CU route (0: never)
    bool single_stream = false;      // run every piece of the QR on the caller's stream (no overlap)
    int accum_panels = 0;            // panels merged per update of the accumulated R (0: by size, 2 below n = 8192 and
                                     // 4 from there on, each measured best there; 1: panel by panel)
    bool fused_whip = true;          // Eq. 4 in the epilogue of the rotation product where the shape allows
    bool heads_batched = true;       // n == 128: all problems of a batch in the same launches
    int split_gemm = 1;              // fp32 products of the derivative from three-plane bf16 splits: 0 never, 1 where the
                                     // shape fits and is large enough to gain, 2 wherever the shape fits
    bool device_sync = true;         // the QR's streams hand over through a device word where a probe allows (else events)
    unsigned long long seq = 0;      // last value handed out for the hand-over words, which only grow
    unsigned long long arrived = 0;  // workgroups counted so far by the one-launch panels' word (zeroed with the status word)
    unsigned long long arrived_rows = 0;   // ... and those below the top block, counted by a word of their own
    int fused_panel = 1;             // tall panels between tall panels as one launch: 0 never, 1 up to fused_panel_rows rows, 2 always
    int two_level_rows = -1;         // blocks of 256 columns with more rows than this defer the update of everything right of
                                     // the next block to ONE product with the block's merged reflector; 0 never, -1 default

    struct Probed { hipStream_t s; bool ok; };
    std::vector<Probed> probed;      // per caller stream: do it and the two internal streams progress independently?
    int objective = DQ_OBJ_WHIP;     // what S4 evaluates (dq_set_objective)
    int quant_bits = 4;
    char* ws = nullptr;
    size_t ws_bytes = 0;
    Profiler prof;
};

namespace {

// ---------------------------------------------------------------- workspace layout
constexpr int kYbRing = 4;    // merged reflector blocks kept at a time (two-level QR)
constexpr int kFarSplit = 4;  // most split-K layers of a deferred update's projection
struct Layout {
    long ld = 0;          // leading dimension of every internal n x n fp32 matrix
    size_t flags = 0, A = 0, R = 0, U = 0, G = 0, B = 0, P = 0, M = 0, tau = 0, Tall = 0, wpart = 0, w2 = 0, wpartB = 0, w2B = 0, qpart = 0, qw = 0, yblk = 0, spart = 0, yring = 0, spartB = 0, wpartF1 = 0, w2F1 = 0, wpartF2 = 0, w2F2 = 0,
           vs = 0, cq = 0, tsl = 0, yall = 0, uinv = 0, uinvo = 0, utmp = 0, x3a = 0, x3b = 0, x3c = 0, x3d = 0, Y = 0, dY = 0, xt = 0, dyt = 0, rbt = 0, losspart = 0, scal = 0, gsplit = 0;
    size_t gsplit_floats = 0;
    size_t total = 0;
};

size_t bump(size_t& cur, size_t bytes) {
    const size_t off = cur;
    cur += (bytes + 255) / 256 * 256;
    return off;
}

Layout make_layout(int n, int T) {
    Layout L;
    L.ld = round_up(n, 8);
    const size_t n2 = (size_t)n * L.ld;
    size_t cur = 0;
    L.flags = bump(cur, 256);
    L.A = bump(cur, n2 * 4);
    L.R = bump(cur, n2 * 4);
    L.U = bump(cur, n2 * 4);
    L.G = bump(cur, n2 * 4);
    L.B = bump(cur, n2 * 4);
    L.P = bump(cur, n2 * 4);
    L.M = bump(cur, n2 * 4);
    L.tau = bump(cur, (size_t)round_up(n, 64) * 4);
    const size_t npanels = (n + kPanel - 1) / kPanel;
    L.Tall = bump(cur, npanels * kPanel * kPanel * 4);
    L.wpart = bump(cur, (size_t)kMaxSplit * kPanel * L.ld * 4);
    L.w2 = bump(cur, (size_t)kPanel * L.ld * 4);
    L.wpartB = bump(cur, (size_t)kMaxSplit * kPanel * L.ld * 4);
    L.w2B = bump(cur, (size_t)kPanel * L.ld * 4);
    L.qpart = bump(cur, (size_t)kMaxSplit * n * kPanel * 4);
    L.qw = bump(cur, (size_t)n * kAccumPanels * kPanel * 4);
    L.yblk = bump(cur, (size_t)n * kAccumPanels * kPanel * 4);
    L.spart = bump(cur, (size_t)(kMaxSplit + 1) * kAccumPanels * kPanel * kPanel * 4);
    // two-level blocking of the QR: a ring of merged reflector blocks Yb = V T (n x 256 each), the merge's partials on the
    // second stream, and the projections of the two deferred updates (256 x ld, up to kFarSplit layers)
    L.yring = bump(cur, (size_t)kYbRing * n * kAccumPanels * kPanel * 4);
    L.spartB = bump(cur, (size_t)(kMaxSplit + 1) * kAccumPanels * kPanel * kPanel * 4);
    L.wpartF1 = bump(cur, (size_t)kFarSplit * kAccumPanels * kPanel * L.ld * 4);
    L.w2F1 = bump(cur, (size_t)kAccumPanels * kPanel * L.ld * 4);
    L.wpartF2 = bump(cur, (size_t)kFarSplit * kAccumPanels * kPanel * L.ld * 4);
    L.w2F2 = bump(cur, (size_t)kAccumPanels * kPanel * L.ld * 4);
    L.vs = bump(cur, panel_scratch_floats(n) * 4);
    L.cq = bump(cur, cholpanel_scratch_floats() * 4);
    L.tsl = bump(cur, (size_t)kPanel * kPanel * 4);
    L.yall = bump(cur, npanels * (size_t)n * kPanel * 4);   // V T of every panel (n x 64 slot each)
    const size_t nblk = (n + kTrsmBlock - 1) / kTrsmBlock;
    L.uinv = bump(cur, nblk * kTrsmBlock * kTrsmBlock * 4);
    L.uinvo = bump(cur, (size_t)round_up(n, kTrsmOuter) * kTrsmOuter * 4);   // inverses of the outer diagonal blocks
    L.utmp = bump(cur, (size_t)round_up(n, kTrsmOuter) * 192 * 4);          // products on the way to them
    // three bf16 planes of up to four n x n operands (fp32 products on the bf16 matrix cores)
    L.x3a = bump(cur, 3 * n2 * 2);
    L.x3b = bump(cur, 3 * n2 * 2);
    L.x3c = bump(cur, 3 * n2 * 2);
    L.x3d = bump(cur, 3 * n2 * 2);
    const size_t tn = (size_t)(T > 0 ? T : 1) * L.ld;
    L.Y = bump(cur, tn * 4);
    L.dY = bump(cur, tn * 4);
    // token-contiguous bf16 copies of X and dY (n x T each) for G = X^T dY
    const size_t tld = (size_t)round_up(T > 0 ? T : 1, 64);
    L.xt = bump(cur, (size_t)round_up(n, 64) * tld * 2);
    L.dyt = bump(cur, (size_t)round_up(n, 64) * tld * 2);
    L.rbt = bump(cur, (size_t)n * 2 * round_up(n, 32) * 2);
    L.losspart = bump(cur, (size_t)kLossPartials * 8);
    L.scal = bump(cur, 256);   // device scalars (the step size of the Cayley update)
    L.gsplit_floats = (size_t)kMaxSplit * n2;
    if (L.gsplit_floats > ((size_t)16 << 20)) L.gsplit_floats = (size_t)16 << 20;
    L.gsplit = bump(cur, L.gsplit_floats * 4);
    L.total = cur;
    return L;
}

template <typename Tp>
Tp* at(dq_ctx* c, size_t off) { return reinterpret_cast<Tp*>(c->ws + off); }

// ---------------------------------------------------------------- argument checks
bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; }

dq_status check_f32(const void* p, long ld, int cols) {
    if (p == nullptr) return DQ_ERR_NULL;
    if (ld < cols) return DQ_ERR_SHAPE;
    if (!aligned16(p) || (ld & 3) != 0) return DQ_ERR_ALIGN;
    return DQ_OK;
}
dq_status check_bf16(const void* p, long ld, int cols) {
    if (p == nullptr) return DQ_ERR_NULL;
    if (ld < cols) return DQ_ERR_SHAPE;
    if (!aligned16(p) || (ld & 7) != 0) return DQ_ERR_ALIGN;
    return DQ_OK;
}
dq_status check_x(const void* p, dq_dtype dt, long ld, int cols) {
    if (dt == DQ_F32) return check_f32(p, ld, cols);
    if (dt == DQ_BF16) return check_bf16(p, ld, cols);
    return DQ_ERR_DTYPE;
}
dq_status check_n(int n) {
    if (n < 1) return DQ_ERR_SHAPE;
    if (n > DQ_MAX_N) return DQ_ERR_UNSUPPORTED;
    return DQ_OK;
}
dq_status check_ws(dq_ctx* c, const Layout& L) {
    if (c->ws == nullptr || c->ws_bytes < L.total) return DQ_ERR_WORKSPACE;
    return DQ_OK;
}

#define DQ_TRY(expr)                      \
    do {                                  \
        const dq_status _s = (expr);      \
        if (_s != DQ_OK) return _s;       \
    } while (0)
#define DQ_HIP(expr)                              \
    do {                                          \
        if ((expr) != hipSuccess) return DQ_ERR_HIP; \
    } while (0)

// ---------------------------------------------------------------- split-K choice
// Enough layers to give every compute unit a workgroup when the output has few tiles.
void choose_split(int tiles, int K, int kalign, int max_splits, int& splits, int& kchunk) {
    constexpr int target = 768;   // workgroups aimed for (three per compute unit)
    constexpr int mink = 128;     // at least this many reduction elements per layer
    splits = 1;
    if (tiles < 256) {
        splits = (target + tiles - 1) / tiles;
        const int by_k = (K + mink - 1) / mink;   // at least `mink` reduction elements per layer
        if (splits > by_k) splits = by_k;
        if (splits > max_splits) splits = max_splits;
        if (splits < 1) splits = 1;
    }
    kchunk = (int)round_up((K + splits - 1) / splits, kalign);
    splits = (K + kchunk - 1) / kchunk;
    if (splits < 1) splits = 1;
}

// ---------------------------------------------------------------- block-reflector application
// Pieces of  Csub <- (I - V op(T) V^T) Csub = Csub - (V op(T)) (V^T Csub)  with V the unit-lower-trapezoid block
// stored at Vp (m x jb, ldv).  Each piece takes the stream and the scratch buffers it may use, so that the look-ahead
// part and the trailing part of a QR update can run on two streams.
struct ReflBufs { float* wpart; float* wsum; };

// Wsum (jb x ncols, ld L.ld) = V^T Bmat;  with gram_cols > 0 the first gram_cols columns of Bmat are V itself (masked).
// a_unit_lower = 0: the left operand is a plain m x jb matrix (V T) instead of the reflector block.
dq_status refl_project(dq_ctx* c, hipStream_t s, const Layout& L, const ReflBufs& bufs, const float* Vp, long ldv,
                       int m, int jb, const float* Bmat, long ldb, int ncols, int gram_cols, const float** Wsum,
                       int max_splits = kMaxSplit, int* splits_out = nullptr, int a_unit_lower = 1) {
    const long ldw = L.ld;
    const long stride = (long)kPanel * ldw;
    int splits, kchunk;
    // A plain left operand (V T) streams best through the 64 x 64 tile configuration (4 workgroups per compute unit);
    // the masked reflector block keeps the shape-chosen one, whose split count the T-factor kernel is sized for.
    const bool small_tiles = !a_unit_lower;
    const int tn = small_tiles ? 64 : gemm_f32_tile_n(jb, ncols);
    choose_split((ncols + tn - 1) / tn, m, small_tiles ? 32 : 16, max_splits, splits, kchunk);
    if (splits_out != nullptr) *splits_out = splits;
    {
        GemmF32 g;
        if (small_tiles) g.cfg = 3;
        g.A = Vp; g.lda = ldv; g.ta = 1; g.a_unit_lower = a_unit_lower;
        g.B = Bmat; g.ldb = ldb; g.tb = 0; g.b_unit_lower_cols = gram_cols;
        g.C = bufs.wpart; g.ldc = ldw;
        g.M = jb; g.N = ncols; g.K = m;
        g.splits = splits; g.kchunk = kchunk; g.split_stride = stride;
        LaunchScope sc(&c->prof, s, DQ_K_GEMM_F32, 2.0 * jb * (double)ncols * m, 0.0);
        DQ_HIP(launch_gemm_f32(g, s));
    }
    *Wsum = bufs.wpart;
    if (splits > 1 && splits_out == nullptr) {   // a caller that asks for the split count sums the partials itself
        LaunchScope sc(&c->prof, s, DQ_K_SMALL, 0.0, 0.0);
        DQ_HIP(launch_splitk_reduce(bufs.wpart, splits, stride, ldw, jb, ncols, 1.f, 0.f, bufs.wsum, ldw, s));
        *Wsum = bufs.wsum;
    }
    return DQ_OK;
}

// Y (m x jb, ld kPanel) = V op(T)
dq_status refl_make_y(dq_ctx* c, hipStream_t s, const float* Vp, long ldv, int m, int jb, const float* Tp, int transT,
                      float* Y) {
    GemmF32 g;
    g.A = Vp; g.lda = ldv; g.ta = 0; g.a_unit_lower = 1;
    g.B = Tp; g.ldb = kPanel; g.tb = transT ? 1 : 0;
    g.C = Y; g.ldc = kPanel;
    g.M = m; g.N = jb; g.K = jb;
    LaunchScope sc(&c->prof, s, DQ_K_GEMM_F32, 2.0 * m * (double)jb * jb, 0.0);
    DQ_HIP(launch_gemm_f32(g, s));
    return DQ_OK;
}

// Csub (m x nc) -= V W  (V: the unit-lower-trapezoid reflector block in the factored matrix, W: jb x nc, ld L.ld)
dq_status refl_update(dq_ctx* c, hipStream_t s, const Layout& L, const float* Vp, long ldv, const float* W, int m,
                      int jb, float* Csub, long ldc, int nc) {
    if (nc <= 0) return DQ_OK;
    GemmF32 g;
    g.A = Vp; g.lda = ldv; g.ta = 0; g.a_unit_lower = 1;
    g.B = W; g.ldb = L.ld; g.tb = 0;
    g.C = Csub; g.ldc = ldc;
    g.M = m; g.N = nc; g.K = jb;
    g.alpha = -1.f; g.beta = 1.f;
    LaunchScope sc(&c->prof, s, DQ_K_GEMM_F32, 2.0 * m * (double)nc * jb, 0.0);
    DQ_HIP(launch_gemm_f32(g, s));
    return DQ_OK;
}

// ---------------------------------------------------------------- S1 + S2
// Q[:, k0:k0+m] <- Q[:, k0:k0+m] (I - V T V^T) for the panel at column k0 (V: m x jb at Vp, Yp = V T: m x jb, ld 64):
//   Wq = Qc Yp (n x jb),  Qc -= Wq V^T.
dq_status accumulate_q(dq_ctx* c, hipStream_t s, const Layout& L, int n, int k0, int m, int jb, const float* Vp,
                       long ldv, const float* Yp, float* Q, long ldq) {
    float* qpart = at<float>(c, L.qpart);
    float* qw = at<float>(c, L.qw);
    float* Qc = Q + k0;
    const long stride = (long)n * kPanel;
    int splits, kchunk;
    const int tm = jb <= 64 ? 256 : 128;
    choose_split((n + tm - 1) / tm, m, 16, kMaxSplit, splits, kchunk);
    {
        GemmF32 g;   // Wq = Qc Yp
        g.A = Qc; g.lda = ldq; g.ta = 0;
        g.B = Yp; g.ldb = kPanel; g.tb = 0;
        g.C = splits > 1 ? qpart : qw; g.ldc = kPanel;
        g.M = n; g.N = jb; g.K = m;
        g.splits = splits; g.kchunk = kchunk; g.split_stride = stride;
        LaunchScope sc(&c->prof, s, DQ_K_GEMM_F32, 2.0 * n * (double)jb * m, 0.0);
        DQ_HIP(launch_gemm_f32(g, s));
    }
    if (splits > 1) {
        LaunchScope sc(&c->prof, s, DQ_K_SMALL, 0.0, 0.0);
        DQ_HIP(launch_splitk_reduce(qpart, splits, stride, kPanel, n, jb, 1.f, 0.f, qw, kPanel, s));
    }
    {
        GemmF32 g;   // Qc -= Wq V^T   (V stored m x jb = N x K)
        g.A = qw; g.lda = kPanel; g.ta = 0;
        g.B = Vp; g.ldb = ldv; g.tb = 1; g.b_unit_lower_cols = jb;
        g.C = Qc; g.ldc = ldq;
        g.M = n; g.N = m; g.K = jb;
        g.alpha = -1.f; g.beta = 1.f;
        LaunchScope sc(&c->prof, s, DQ_K_GEMM_F32, 2.0 * n * (double)m * jb, 0.0);
        DQ_HIP(launch_gemm_f32(g, s));
    }
    return DQ_OK;
}

// The same for a run of np consecutive panels (first one q0) at once: their block reflectors are merged into one of
// width w = sum of the panel widths,  H_q0 ... H_(q0+np-1) = I - V Yb^T... in the form used here
//   Q[:, k0:] <- Q[:, k0:] - (Q[:, k0:] Yb) V^T,
// with V the unit-lower-trapezoid block of the w columns and Yb = V T_merged built column group by column group:
//   Yb_j = [0; Yp_j] - Yb_{<j} (V_{<j}^T [0; Yp_j]).
// A K = 256 update reads and writes the accumulated factor once per four panels instead of once per panel (the
// K = 64 update is bound by that traffic), for a few small products more.
// (merge_yb_step builds one column group of Yb, accumulate_q_apply applies a merged block; the two-level QR uses both.)
// One column group of the merged block: panel q0 + j of the block that starts at panel q0 goes into Yb (ld 256).
dq_status merge_yb_step(dq_ctx* c, hipStream_t s, int n, int nb, int q0, int j, float* A, long ld, float* yall,
                        float* Yb, float* spart) {
    const int k0 = q0 * nb;
    const int mb = n - k0;
    float* Ablk = A + (long)k0 * ld + k0;
    const long ldy = (long)kAccumPanels * kPanel;
    float* sred = spart + (size_t)kMaxSplit * kAccumPanels * kPanel * kPanel;
    const int q = q0 + j;
    const int off = q * nb - k0;
    const int mq = n - q * nb;
    const int jq = mq < nb ? mq : nb;
    const float* Ypq = yall + (long)q * n * kPanel;
    {
        LaunchScope sc(&c->prof, s, DQ_K_SMALL, 0.0, 8.0 * mb * (double)jq);
        if (off > 0) DQ_HIP(launch_copy2d(nullptr, 0, Yb + off, ldy, off, jq, s));
        DQ_HIP(launch_copy2d(Ypq, kPanel, Yb + (long)off * ldy + off, ldy, mq, jq, s));
    }
    if (j > 0) {
        // S = V_{<j}^T [0; Yp_j]: only rows >= off of V_{<j} meet non-zeros, all of them below its diagonal
        int splits, kchunk;
        choose_split(((off + 63) / 64) * ((jq + 63) / 64), mq, 32, kMaxSplit, splits, kchunk);
        const long stride = (long)kAccumPanels * kPanel * kPanel;
        {
            GemmF32 g;
            g.cfg = 3;
            g.A = Ablk + (long)off * ld; g.lda = ld; g.ta = 1;
            g.B = Ypq; g.ldb = kPanel; g.tb = 0;
            g.C = splits > 1 ? spart : sred; g.ldc = kPanel;
            g.M = off; g.N = jq; g.K = mq;
            g.splits = splits; g.kchunk = kchunk; g.split_stride = stride;
            LaunchScope sc(&c->prof, s, DQ_K_GEMM_F32, 2.0 * off * (double)jq * mq, 0.0);
            DQ_HIP(launch_gemm_f32(g, s));
        }
        if (splits > 1) {
            LaunchScope sc(&c->prof, s, DQ_K_SMALL, 0.0, 0.0);
            DQ_HIP(launch_splitk_reduce(spart, splits, stride, kPanel, off, jq, 1.f, 0.f, sred, kPanel, s));
        }
        {
            GemmF32 g;   // Yb_j -= Yb_{<j} S
            g.A = Yb; g.lda = ldy; g.ta = 0;
            g.B = sred; g.ldb = kPanel; g.tb = 0;
            g.C = Yb + off; g.ldc = ldy;
            g.M = mb; g.N = jq; g.K = off;
            g.alpha = -1.f; g.beta = 1.f;
            LaunchScope sc(&c->prof, s, DQ_K_GEMM_F32, 2.0 * mb * (double)jq * off, 0.0);
            DQ_HIP(launch_gemm_f32(g, s));
        }
    }
    return DQ_OK;
}

// Q[:, k0:] <- Q[:, k0:] - (Q[:, k0:] Yb) V^T for a merged block of width w whose top-left corner is (k0, k0).
dq_status accumulate_q_apply(dq_ctx* c, hipStream_t s, const Layout& L, int n, int k0, int w, float* A, long ld,
                             const float* Yb, float* Q, long ldq) {
    const int mb = n - k0;
    float* Ablk = A + (long)k0 * ld + k0;
    const long ldy = (long)kAccumPanels * kPanel;
    float* qpart = at<float>(c, L.qpart);
    float* qw = at<float>(c, L.qw);
    float* Qc = Q + k0;
    const long stride = (long)n * ldy;
    int splits, kchunk;
    int max_splits = (int)(((size_t)kMaxSplit * n * kPanel) / ((size_t)n * ldy));   // what the partial buffer holds
    if (max_splits < 1) max_splits = 1;
    choose_split(((n + 127) / 128) * ((w + 127) / 128), mb, 16, max_splits, splits, kchunk);
    {
        GemmF32 g;   // Wq = Qc Yb
        g.A = Qc; g.lda = ldq; g.ta = 0;
        g.B = Yb; g.ldb = ldy; g.tb = 0;
        g.C = splits > 1 ? qpart : qw; g.ldc = ldy;
        g.M = n; g.N = w; g.K = mb;
        g.splits = splits; g.kchunk = kchunk; g.split_stride = stride;
        LaunchScope sc(&c->prof, s, DQ_K_GEMM_F32, 2.0 * n * (double)w * mb, 0.0);
        DQ_HIP(launch_gemm_f32(g, s));
    }
    if (splits > 1) {
        LaunchScope sc(&c->prof, s, DQ_K_SMALL, 0.0, 0.0);
        DQ_HIP(launch_splitk_reduce(qpart, splits, stride, ldy, n, w, 1.f, 0.f, qw, ldy, s));
    }
    {
        GemmF32 g;   // Qc -= Wq V^T   (V stored mb x w = N x K)
        g.A = qw; g.lda = ldy; g.ta = 0;
        g.B = Ablk; g.ldb = ld; g.tb = 1; g.b_unit_lower_cols = w;
        g.C = Qc; g.ldc = ldq;
        g.M = n; g.N = mb; g.K = w;
        g.alpha = -1.f; g.beta = 1.f;
        LaunchScope sc(&c->prof, s, DQ_K_GEMM_F32, 2.0 * n * (double)mb * w, 0.0);
        DQ_HIP(launch_gemm_f32(g, s));
    }
    return DQ_OK;
}

dq_status accumulate_q_block(dq_ctx* c, hipStream_t s, const Layout& L, int n, int nb, int q0, int np, float* A, long ld,
                             float* yall, float* Q, long ldq) {
    float* Yb = at<float>(c, L.yblk);
    int w = 0;
    for (int j = 0; j < np; ++j) {
        DQ_TRY(merge_yb_step(c, s, n, nb, q0, j, A, ld, yall, Yb, at<float>(c, L.spart)));
        const int mq = n - (q0 + j) * nb;
        w += mq < nb ? mq : nb;
    }
    return accumulate_q_apply(c, s, L, n, q0 * nb, w, A, ld, Yb, Q, ldq);
}

// The block reflector of a merged block (w columns from (k0, k0); Yb = V T, ld 256) applied to the columns
// [c0, c0 + nc) of the factored matrix:  W = Yb^T C,  C -= V W, with reduction length w in the second product.
dq_status far_update(dq_ctx* c, hipStream_t s, const Layout& L, float* wpart, float* wsum, int n, int k0, int w,
                     float* A, long ld, const float* Yb, int c0, int nc) {
    if (nc <= 0) return DQ_OK;
    const int mb = n - k0;
    const long ldy = (long)kAccumPanels * kPanel;
    const long ldw = L.ld;
    const long stride = (long)kAccumPanels * kPanel * ldw;
    float* Ablk = A + (long)k0 * ld + k0;
    float* Cf = A + (long)k0 * ld + c0;
    int splits, kchunk;
    choose_split(((w + 127) / 128) * ((nc + 127) / 128), mb, 16, kFarSplit, splits, kchunk);
    {
        GemmF32 g;   // W = Yb^T C
        g.A = Yb; g.lda = ldy; g.ta = 1;
        g.B = Cf; g.ldb = ld; g.tb = 0;
        g.C = splits > 1 ? wpart : wsum; g.ldc = ldw;
        g.M = w; g.N = nc; g.K = mb;
        g.splits = splits; g.kchunk = kchunk; g.split_stride = stride;
        LaunchScope sc(&c->prof, s, DQ_K_GEMM_F32, 2.0 * w * (double)nc * mb, 0.0);
        DQ_HIP(launch_gemm_f32(g, s));
    }
    if (splits > 1) {
        LaunchScope sc(&c->prof, s, DQ_K_SMALL, 0.0, 0.0);
        DQ_HIP(launch_splitk_reduce(wpart, splits, stride, ldw, w, nc, 1.f, 0.f, wsum, ldw, s));
    }
    return refl_update(c, s, L, Ablk, ld, wsum, mb, w, Cf, ld, nc);
}

// ---------------------------------------------------------------- hand-over between the QR's streams
// Seven 8-byte words behind the status word, cleared with it: [0] panels factored, [1] trailing updates done,
// [2] the probe's word, [3] set by a probe wait that gave up, [4..6] the words of the one-launch panels
// (launch_cholqr_fused).
constexpr long kSyncLimitUs = 5L * 1000 * 1000;   // a hand-over that takes this long is a fault, not a delay
constexpr long kProbeLimitUs = 2000;
constexpr int kFusedPanelRows = 8192;   // tallest panel that takes the one-launch route by default
constexpr int kTwoLevelRows = 2048;     // blocks of 256 columns taller than this take the two-level route by default ...
constexpr int kTwoLevelMinN = 6144;     // ... in matrices of at least this order (measured: 8192 27.7 -> 26.0 ms; 5120 and
                                        // 4096, where the panel chain and not the rank-64 updates sets the pace: +-1 %, +3 %)
unsigned long long* sync_words(dq_ctx* c) { return reinterpret_cast<unsigned long long*>(c->ws + 128); }

// Device-side hand-over needs the consumer's wait kernel and the producer's signal kernel to run at the same time.
// Streams that share a hardware queue cannot (the wait would sit in front of the signal), and inside a stream
// capture the order of execution is not ours: both cases take the event route.  Probed once per caller stream: a
// bounded wait on each consuming stream, the signal on its producer enqueued AFTER it.
// Is a bounded wait enqueued on `consumer` released by a signal enqueued AFTER it on `producer`?  Both streams are idle
// when this returns.
hipError_t handover_probe(dq_ctx* c, hipStream_t consumer, hipStream_t producer, bool* usable) {
    unsigned long long* w = sync_words(c);
    const unsigned long long v = ++c->seq;
    hipError_t e;
    if ((e = launch_stream_wait(w + 2, v, kProbeLimitUs, nullptr, w + 3, consumer)) != hipSuccess) return e;
    if ((e = launch_stream_signal(w + 2, v, producer)) != hipSuccess) return e;
    if ((e = hipStreamSynchronize(consumer)) != hipSuccess) return e;
    if ((e = hipStreamSynchronize(producer)) != hipSuccess) return e;
    unsigned long long gave_up = 1;
    if ((e = hipMemcpy(&gave_up, w + 3, sizeof(gave_up), hipMemcpyDeviceToHost)) != hipSuccess) return e;
    *usable = gave_up == 0;
    if (gave_up != 0) {
        if ((e = launch_fill_u32(reinterpret_cast<unsigned*>(w + 3), 2, 0u, consumer)) != hipSuccess) return e;
        if ((e = hipStreamSynchronize(consumer)) != hipSuccess) return e;
    }
    return hipSuccess;
}

bool device_sync_usable(dq_ctx* c) {
    if (!c->device_sync || c->single_stream) return false;
    for (const dq_ctx::Probed& pr : c->probed)
        if (pr.s == c->stream) return pr.ok;
    hipStreamCaptureStatus cs = hipStreamCaptureStatusNone;
    if (hipStreamIsCapturing(c->stream, &cs) != hipSuccess || cs != hipStreamCaptureStatusNone) {
        (void)hipGetLastError();
        return false;
    }
    bool ok = hipStreamSynchronize(c->stream) == hipSuccess;   // the probe must not sit behind the caller's backlog
    hipStream_t pairs[3][2] = {{c->stream2, c->stream}, {c->stream3, c->stream}, {c->stream, c->stream2}};   // {consumer, producer}
    for (int i = 0; i < 3 && ok; ++i) {
        bool usable = false;
        ok = handover_probe(c, pairs[i][0], pairs[i][1], &usable) == hipSuccess && usable;
    }
    c->probed.push_back({c->stream, ok});
    return ok;
}

dq_status qr_orth_one(dq_ctx* c, const Layout& L, int n, const float* Z, long ldz, float* R, long ldr, float* U,
                      long ldu) {
    hipStream_t sA = c->stream, sB = c->single_stream ? c->stream : c->stream2,
                sC = c->single_stream ? c->stream : c->stream3;
    float* A = at<float>(c, L.A);
    float* tau = at<float>(c, L.tau);
    float* Tall = at<float>(c, L.Tall);
    float* vs = at<float>(c, L.vs);
    float* tsl = at<float>(c, L.tsl);
    float* yall = at<float>(c, L.yall);
    unsigned* flags = at<unsigned>(c, L.flags);
    const ReflBufs bufA{at<float>(c, L.wpart), at<float>(c, L.w2)};
    const long ld = L.ld;
    // how the streams wait for each other: a device word (see device_sync_usable) or events
    const bool dsync = device_sync_usable(c);
    unsigned long long* words = sync_words(c);
    const unsigned long long seq0 = c->seq;
    auto panel_done = [&](int p) -> hipError_t {            // on sA: panel p is factored
        return dsync ? launch_stream_signal(words, seq0 + p + 1, sA) : hipEventRecord(c->sync_ev[2 * p], sA);
    };
    auto after_panel = [&](hipStream_t s, int p) -> hipError_t {   // s goes on once panel p is factored
        return dsync ? launch_stream_wait(words, seq0 + p + 1, kSyncLimitUs, flags, nullptr, s)
                     : hipStreamWaitEvent(s, c->sync_ev[2 * p], 0);
    };
    auto trailing_done = [&](int p) -> hipError_t {         // on sB: the trailing update of panel p has run
        return dsync ? launch_stream_signal(words + 1, seq0 + p + 1, sB) : hipEventRecord(c->sync_ev[2 * p + 1], sB);
    };
    auto after_trailing = [&](int p) -> hipError_t {        // sA goes on once the trailing update of panel p has run
        return dsync ? launch_stream_wait(words + 1, seq0 + p + 1, kSyncLimitUs, flags, nullptr, sA)
                     : hipStreamWaitEvent(sA, c->sync_ev[2 * p + 1], 0);
    };
    {
        LaunchScope sc(&c->prof, sA, DQ_K_SMALL, 0.0, 8.0 * n * (double)n);
        DQ_HIP(launch_copy2d(Z, ldz, A, ld, n, n, sA));
        DQ_HIP(launch_set_identity(R, ldr, n, sA));
    }
    if (dsync) {
        // The polls are bounded, and bounded for THIS call's work: the internal streams only begin to poll once the
        // caller's stream has reached this call, however much the caller had enqueued in front of it.
        DQ_HIP(hipEventRecord(c->sync_ev[0], sA));
        DQ_HIP(hipStreamWaitEvent(sB, c->sync_ev[0], 0));
        DQ_HIP(hipStreamWaitEvent(sC, c->sync_ev[0], 0));
    }
    // S1.  Panel p is factored on the caller's stream while the trailing update of panel p-1 still runs on the
    // second stream: after panel p only the columns of panel p+1 ("look-ahead" part) are updated on the caller's
    // stream; the rest of the trailing matrix goes to the second stream.
    const int nb = kPanel;
    const int npanels = (n + nb - 1) / nb;
    c->seq += npanels + 1;
    int last_trailing = -1;
    bool gram_ready = false;   // the first small step of the coming panel (chol of its Gram matrix) was done beside the previous panel's look-ahead
    // Two-level blocking for the tall part of a large matrix: in a block of 256 columns (four panels) each panel's
    // reflector only reaches the 256 + 64 columns after the block's start on the second stream ("near"); everything
    // right of that receives ONE update per block with the block's merged reflector, reduction length 256 instead of 64
    // (a quarter of the passes over the trailing matrix): first the columns the next block's panels need ("far-near",
    // second stream, signals word F), then the rest ("far-rest", third stream in front of the accumulation of R, which
    // uses the same merged block; signals F2; the accumulation F3, which frees the block's slot in the ring of merged
    // blocks).  The panel chain runs on across block boundaries: a block's first panel waits for F of the block before.
    const int ob = kAccumPanels * kPanel;
    const int two_rows = c->two_level_rows < 0 ? (n >= kTwoLevelMinN ? kTwoLevelRows : 0) : c->two_level_rows;
    int tl_blocks = 0;
    if (dsync && !c->single_stream && two_rows > 0 && n % ob == 0 && c->chol_min_m > 0 && c->chol_min_m <= 4 * nb)
        while ((tl_blocks + 1) * ob < n && n - tl_blocks * ob > two_rows) ++tl_blocks;
    unsigned long long* wF = words + 11;    // far-near of block b done: seq0 + b + 1
    unsigned long long* wF2 = words + 12;   // far-rest of block b done
    unsigned long long* wF3 = words + 13;   // accumulation of block b done
    const ReflBufs bufB{at<float>(c, L.wpartB), at<float>(c, L.w2B)};
    float* yring = at<float>(c, L.yring);
    for (int p = 0; p < npanels; ++p) {
        const int k0 = p * nb;
        const int jb = (n - k0) < nb ? (n - k0) : nb;
        const int m = n - k0;
        float* Ap = A + (long)k0 * ld + k0;
        float* Tp = Tall + (long)p * kPanel * kPanel;
        float* Yp = yall + (long)p * n * kPanel;
        const int nla = (m - jb) < nb ? (m - jb) : nb;
        // Tall full-width panels: CholeskyQR2 + Householder reconstruction over many compute units; it returns the
        // reflectors, T and Yp = V T.  The other panels: the one-workgroup Householder panel kernel, then T from the
        // Gram matrix of the reflectors.
        const bool tall = c->chol_min_m > 0 && m >= c->chol_min_m && cholpanel_supported(Ap, ld, m, jb);
        bool signalled = false;   // "panel p is factored" already goes out from inside the panel's kernels
        const bool two = p < kAccumPanels * tl_blocks;          // this panel's block takes the two-level route
        const int blk = p / kAccumPanels, jblk = p % kAccumPanels;
        const int K0 = blk * ob;
        // what the look-ahead columns (and, without the fused look-ahead, the kernels that read them) wait for: the
        // previous trailing update, or, behind a two-level block, that block's far-near update
        const bool after_block = tl_blocks > 0 && jblk == 0 && blk > 0 && blk <= tl_blocks;
        const unsigned long long* la_word = after_block ? wF : (last_trailing >= 0 ? words + 1 : nullptr);
        const unsigned long long la_value = after_block ? seq0 + blk : seq0 + last_trailing + 1;
        if (tall) {
            // the look-ahead update of the next panel's columns is fused into the last two kernels of the route when
            // that panel is a full one; they also leave the Cholesky factor of the Gram matrix the next tall panel starts from
            const int m2 = m - jb;
            const bool fused_la = nla == kPanel;
            const bool next_tall = fused_la && m2 >= c->chol_min_m &&
                                   cholpanel_supported(Ap + (long)jb * ld + jb, ld, m2, m2 < nb ? m2 : nb);
            // ... and between two such panels the whole route is one launch whose workgroups hand over to each other
            const int fused_wgs = (dsync && gram_ready && fused_la && next_tall && c->fused_panel != 0 &&
                                   (c->fused_panel == 2 || m <= kFusedPanelRows))
                                      ? cholqr_fused_workgroups(m) : 0;
            if (fused_wgs > 0) {
                HandOver ho;
                if (la_word != nullptr) {
                    ho.wait_word = la_word; ho.wait_value = la_value;
                    ho.limit_us = kSyncLimitUs; ho.flags = flags;
                }
                ho.signal_word = words; ho.signal_value = seq0 + p + 1;
                signalled = true;
                c->arrived += (unsigned long long)fused_wgs;
                c->arrived_rows += (unsigned long long)(fused_wgs - 1);
                LaunchScope sc(&c->prof, sA, DQ_K_PANEL, 2.0 * m * (double)jb * jb + 4.0 * m * (double)jb * nla, 0.0);
                DQ_HIP(launch_cholqr_fused(Ap, ld, m, Tp, Yp, vs, at<float>(c, L.cq), tau + k0, tsl, flags, words + 4,
                                           seq0 + p + 1, c->arrived, c->arrived_rows, kSyncLimitUs, sA, &ho));
                gram_ready = true;
            } else {
            {
                LaunchScope sc(&c->prof, sA, DQ_K_PANEL, 2.0 * m * (double)jb * jb, 0.0);
                DQ_HIP(launch_cholqr_factor(Ap, ld, m, Tp, Yp, vs, at<float>(c, L.cq), tau + k0, tsl, flags,
                                            gram_ready ? 1 : 0, sA));
            }
            // the look-ahead columns received update p-1 on the second stream.  With the device-side hand-over and the
            // fused look-ahead, the wait sits at the start of the kernel that first reads those columns and the signal
            // "panel p is factored" at the start of the kernel after it: no launch of their own on the critical path.
            HandOver ho;
            signalled = dsync && fused_la;
            if (signalled) {
                if (la_word != nullptr) {
                    ho.wait_word = la_word; ho.wait_value = la_value;
                    ho.limit_us = kSyncLimitUs; ho.flags = flags;
                }
                ho.signal_word = words; ho.signal_value = seq0 + p + 1;
            } else if (last_trailing >= 0) {
                DQ_HIP(after_trailing(last_trailing));
            }
            {
                LaunchScope sc(&c->prof, sA, DQ_K_PANEL, 4.0 * m * (double)jb * nla, 0.0);
                DQ_HIP(launch_cholqr_finish(Ap, ld, m, Yp, vs, at<float>(c, L.cq), fused_la ? 1 : 0, next_tall ? 1 : 0, flags,
                                            sA, signalled ? &ho : nullptr));
            }
            gram_ready = next_tall;
            if (!fused_la && nla > 0) {   // C_la -= V (Yp^T C_la)
                const float* Wa = nullptr;
                DQ_TRY(refl_project(c, sA, L, bufA, Yp, kPanel, m, jb, Ap + jb, ld, nla, 0, &Wa, kMaxSplit, nullptr, 0));
                DQ_TRY(refl_update(c, sA, L, Ap, ld, Wa, m, jb, Ap + jb, ld, nla));
            }
            }
        } else {
            gram_ready = false;
            int sw = 8;
            {
                LaunchScope sc(&c->prof, sA, DQ_K_PANEL, 2.0 * m * (double)jb * jb, 0.0);
                DQ_HIP(launch_qr_panel(Ap, ld, m, jb, tau + k0, vs, tsl, &sw, flags, sA));
            }
            if (last_trailing >= 0) DQ_HIP(after_trailing(last_trailing));
            // partials of V^T [V | C_la]; summed inside the T-factor kernel, which also returns W2 = T^T V^T C_la
            const float* Wa = nullptr;
            int splitsA = 1;
            DQ_TRY(refl_project(c, sA, L, bufA, Ap, ld, m, jb, Ap, ld, jb + nla, jb, &Wa, 16, &splitsA));
            {
                LaunchScope sc(&c->prof, sA, DQ_K_SMALL, 0.0, 0.0);
                DQ_HIP(launch_tfactor(bufA.wpart, splitsA, (long)kPanel * ld, ld, jb, nla, tsl, sw, Tp, bufA.wsum, sA));
            }
            if (nla > 0) {
                GemmF32 g;   // C_la -= V W2
                g.A = Ap; g.lda = ld; g.ta = 0; g.a_unit_lower = 1;
                g.B = bufA.wsum; g.ldb = kPanel; g.tb = 0;
                g.C = Ap + jb; g.ldc = ld;
                g.M = m; g.N = nla; g.K = jb;
                g.alpha = -1.f; g.beta = 1.f;
                LaunchScope sc(&c->prof, sA, DQ_K_GEMM_F32, 2.0 * m * (double)nla * jb, 0.0);
                DQ_HIP(launch_gemm_f32(g, sA));
            }
            DQ_TRY(refl_make_y(c, sA, Ap, ld, m, jb, Tp, 0, Yp));
        }
        // one level: everything right of the look-ahead columns; two levels: up to 64 columns into the next block
        int rest = m - jb - nla;
        if (two) rest = (K0 + ob + nb < n ? K0 + ob + nb : n) - (k0 + jb + nla);
        if (rest < 0) rest = 0;
        if (!signalled) DQ_HIP(panel_done(p));
        if (rest > 0 || two) DQ_HIP(after_panel(sB, p));
        if (rest > 0) {   // C -= V (Yp^T C) for the rest of the trailing matrix, behind the next panel
            // the first panel behind the two-level blocks updates columns that the last block's far-rest update reaches
            if (!two && tl_blocks > 0 && p == kAccumPanels * tl_blocks)
                DQ_HIP(launch_stream_wait(wF2, seq0 + tl_blocks, kSyncLimitUs, flags, nullptr, sB));
            const float* Wb = nullptr;
            DQ_TRY(refl_project(c, sB, L, bufB, Yp, kPanel, m, jb, Ap + jb + nla, ld, rest, 0, &Wb, kMaxSplit, nullptr, 0));
            DQ_TRY(refl_update(c, sB, L, Ap, ld, Wb, m, jb, Ap + jb + nla, ld, rest));
            DQ_HIP(trailing_done(p));
            last_trailing = p;
        }
        // S2, overlapped with the factorisation of the next panels: the orthogonal factor is accumulated from the
        // left to the right, Q[:, k0:] <- Q[:, k0:] (I - V T V^T)  (as Alg. 2 does column by column), on the third
        // stream, several panels at a time.
        if (two) {
            // this panel's column group of the block's merged reflector, on the second stream behind its near update;
            // the slot of the ring is free once the accumulation of the block that used it last has run
            float* Yb = yring + (size_t)(blk % kYbRing) * n * ob;
            if (jblk == 0 && blk >= kYbRing)
                DQ_HIP(launch_stream_wait(wF3, seq0 + blk - kYbRing + 1, kSyncLimitUs, flags, nullptr, sB));
            DQ_TRY(merge_yb_step(c, sB, n, nb, blk * kAccumPanels, jblk, A, ld, yall, Yb, at<float>(c, L.spartB)));
            if (jblk == kAccumPanels - 1) {
                const int c1 = K0 + ob + nb;                              // first column the near updates did not reach
                const int c2 = (c1 + ob) < n ? (c1 + ob) : n;             // far-near: what the next block's panels touch
                // far-near needs the far-rest update of the block before on its columns
                if (blk > 0) DQ_HIP(launch_stream_wait(wF2, seq0 + blk, kSyncLimitUs, flags, nullptr, sB));
                DQ_TRY(far_update(c, sB, L, at<float>(c, L.wpartF1), at<float>(c, L.w2F1), n, K0, ob, A, ld, Yb, c1, c2 - c1));
                DQ_HIP(launch_stream_signal(wF, seq0 + blk + 1, sB));
                DQ_HIP(launch_stream_wait(wF, seq0 + blk + 1, kSyncLimitUs, flags, nullptr, sC));
                DQ_TRY(far_update(c, sC, L, at<float>(c, L.wpartF2), at<float>(c, L.w2F2), n, K0, ob, A, ld, Yb, c2, n - c2));
                DQ_HIP(launch_stream_signal(wF2, seq0 + blk + 1, sC));
                DQ_TRY(accumulate_q_apply(c, sC, L, n, K0, ob, A, ld, Yb, R, ldr));
                DQ_HIP(launch_stream_signal(wF3, seq0 + blk + 1, sC));
            }
        }
        const int ap = c->accum_panels > 0 ? c->accum_panels : (n >= 8192 ? 4 : 2);
        if (!two && ((p + 1) % ap == 0 || p == npanels - 1)) {
            const int q0 = (p / ap) * ap;
            DQ_HIP(after_panel(sC, p));
            if (p - q0 + 1 == 1)
                DQ_TRY(accumulate_q(c, sC, L, n, k0, m, jb, Ap, ld, Yp, R, ldr));
            else
                DQ_TRY(accumulate_q_block(c, sC, L, n, nb, q0, p - q0 + 1, A, ld, yall, R, ldr));
        }
    }
    if (last_trailing >= 0) DQ_HIP(after_trailing(last_trailing));
    DQ_HIP(hipEventRecord(c->sync_ev.back(), sC));
    DQ_HIP(hipStreamWaitEvent(sA, c->sync_ev.back(), 0));
    {
        LaunchScope sc(&c->prof, sA, DQ_K_SMALL, 0.0, 12.0 * n * (double)n);
        DQ_HIP(launch_sign_normalise(A, ld, n, R, ldr, U, ldu, flags, sA));
    }
    return DQ_OK;
}

// ---------------------------------------------------------------- S3 + S4 + S5
dq_status rotate_loss_grad_one(dq_ctx* c, const Layout& L, int T, int n, const void* X, dq_dtype xdt, long ldx,
                               const float* R, long ldr, dq_reduce red, float* loss_dev, float* G, long ldg,
                               float* Y, long ldy, void* dY, long lddy, bool keep_y_dy = true) {
    hipStream_t s = c->stream;
    unsigned* flags = at<unsigned>(c, L.flags);
    double* lpart = at<double>(c, L.losspart);
    const float scale = (red == DQ_REDUCE_TOKEN_MEAN) ? 1.f / (float)T : 1.f;
    const double gemm_flops = 2.0 * T * (double)n * n;
    const bool use_fused = c->fused_whip;
    // large round bf16 shapes: S5 reads token-contiguous copies of both operands (see below)
    const bool g_transposed = xdt == DQ_BF16 && n % 128 == 0 && T % 128 == 0 && (n / 128) * (n / 128) >= 256 &&
                              (ldx & 7) == 0 && aligned16(X) && aligned16(G) && (ldg & 3) == 0;
    bool fused = false;   // S4 done in the epilogue of S3
    // S3: Y = X @ R
    if (xdt == DQ_BF16) {
        bf16_t* rbt = at<bf16_t>(c, L.rbt);
        // R enters the bf16 matrix cores as two planes, R = hi + lo (16 mantissa bits), so that the rotation
        // keeps close to fp32 accuracy: Y = X @ hi + X @ lo in one pass over the accumulators.
        const int koff = (int)round_up(n, 32);
        {
            LaunchScope sc(&c->prof, s, DQ_K_SMALL, 0.0, 8.0 * n * (double)n);
            DQ_HIP(launch_split_transpose_bf16(R, ldr, n, rbt, 2L * koff, koff, s));
        }
        GemmBf16 g;
        g.A = static_cast<const bf16_t*>(X); g.lda = ldx; g.ta = 0;
        g.B = rbt; g.ldb = 2L * koff; g.tb = 1;
        g.C = Y; g.ldc = ldy; g.M = T; g.N = n; g.K = 2 * koff;
        g.a_kwrap = koff; g.a_klim = n;
        // A caller that needs neither Y nor dY gets Eq. 4 and its derivative applied to the accumulators: Y is never
        // written and dY leaves the kernel already transposed for S5.
        fused = use_fused && !keep_y_dy && g_transposed && gemm_bf16_deep_fits(g) && c->objective == DQ_OBJ_WHIP &&
                gemm_bf16_whip_partials(g) <= kLossPartials;
        if (fused) {
            g.C = nullptr;
            g.whip_dyt = at<bf16_t>(c, L.dyt); g.whip_ldt = T; g.whip_scale = scale; g.whip_partials = lpart;
        }
        {
            LaunchScope sc(&c->prof, s, DQ_K_GEMM_BF16, gemm_flops, 0.0);
            DQ_HIP(launch_gemm_bf16(g, s));
        }
        if (fused) {
            LaunchScope sc(&c->prof, s, DQ_K_SMALL, 0.0, 0.0);
            DQ_HIP(launch_loss_finish(lpart, gemm_bf16_whip_partials(g), scale, loss_dev, flags, s));
        }
    } else {
        GemmF32 g;
        g.A = static_cast<const float*>(X); g.lda = ldx; g.ta = 0;
        g.B = R; g.ldb = ldr; g.tb = 0;
        g.C = Y; g.ldc = ldy; g.M = T; g.N = n; g.K = n;
        LaunchScope sc(&c->prof, s, DQ_K_GEMM_F32, gemm_flops, 0.0);
        DQ_HIP(launch_gemm_f32(g, s));
    }
    // S4: loss and dY in one pass over Y
    if (!fused) {
        const bool whip = c->objective == DQ_OBJ_WHIP;
        const int grid = whip ? whip_grid(T, n) : objective_grid(T, n);
        const double bytes = (double)T * n * (4.0 + (xdt == DQ_BF16 ? 2.0 : 4.0));
        {
            LaunchScope sc(&c->prof, s, DQ_K_WHIP, 5.0 * T * (double)n, bytes);
            if (whip) DQ_HIP(launch_whip(Y, ldy, T, n, scale, dY, xdt == DQ_BF16, lddy, lpart, grid, s));
            else DQ_HIP(launch_objective(c->objective, c->quant_bits, Y, ldy, T, n, scale, dY, xdt == DQ_BF16, lddy,
                                         lpart, grid, s));
        }
        LaunchScope sc(&c->prof, s, DQ_K_SMALL, 0.0, 0.0);
        DQ_HIP(launch_loss_finish(lpart, grid, scale, loss_dev, flags, s));
    }
    // S5: G = X^T @ dY (reduction over the tokens; split when the n x n output has few tiles)
    {
        const int tiles = ((n + 127) / 128) * ((n + 127) / 128);
        int max_splits = (int)(L.gsplit_floats / ((size_t)n * L.ld));
        if (max_splits > kMaxSplit) max_splits = kMaxSplit;
        if (max_splits < 1) max_splits = 1;
        int splits, kchunk;
        choose_split(tiles, T, 32, max_splits, splits, kchunk);
        float* gs = at<float>(c, L.gsplit);
        float* out = splits > 1 ? gs : G;
        const long ldo = splits > 1 ? L.ld : ldg;
        const long stride = (long)n * L.ld;
        // Large round bf16 shapes: both operands are first transposed (two HBM-bound passes), so that the product
        // reads rows only and runs in the unguarded deep-prefetch kernel without a split of the token sum.
        if (g_transposed && (fused || ((lddy & 7) == 0 && aligned16(dY)))) {
            bf16_t* xt = at<bf16_t>(c, L.xt);
            bf16_t* dyt = at<bf16_t>(c, L.dyt);
            {
                LaunchScope sc(&c->prof, s, DQ_K_SMALL, 0.0, (fused ? 4.0 : 8.0) * T * (double)n);
                DQ_HIP(launch_transpose_bf16(static_cast<const bf16_t*>(X), ldx, T, n, xt, T, s));
                if (!fused) DQ_HIP(launch_transpose_bf16(static_cast<const bf16_t*>(dY), lddy, T, n, dyt, T, s));
            }
            GemmBf16 g;
            g.A = xt; g.lda = T; g.ta = 0;
            g.B = dyt; g.ldb = T; g.tb = 1;
            g.C = G; g.ldc = ldg; g.M = n; g.N = n; g.K = T;
            LaunchScope sc(&c->prof, s, DQ_K_GEMM_BF16, gemm_flops, 0.0);
            DQ_HIP(launch_gemm_bf16(g, s));
            return DQ_OK;
        }
        if (xdt == DQ_BF16) {
            GemmBf16 g;
            g.A = static_cast<const bf16_t*>(X); g.lda = ldx; g.ta = 1;
            g.B = static_cast<const bf16_t*>(dY); g.ldb = lddy; g.tb = 0;
            g.C = out; g.ldc = ldo; g.M = n; g.N = n; g.K = T;
            g.splits = splits; g.kchunk = kchunk; g.split_stride = stride;
            LaunchScope sc(&c->prof, s, DQ_K_GEMM_BF16, gemm_flops, 0.0);
            DQ_HIP(launch_gemm_bf16(g, s));
        } else {
            GemmF32 g;
            g.A = static_cast<const float*>(X); g.lda = ldx; g.ta = 1;
            g.B = static_cast<const float*>(dY); g.ldb = lddy; g.tb = 0;
            g.C = out; g.ldc = ldo; g.M = n; g.N = n; g.K = T;
            g.splits = splits; g.kchunk = kchunk; g.split_stride = stride;
            LaunchScope sc(&c->prof, s, DQ_K_GEMM_F32, gemm_flops, 0.0);
            DQ_HIP(launch_gemm_f32(g, s));
        }
        if (splits > 1) {
            LaunchScope sc(&c->prof, s, DQ_K_SMALL, 0.0, 0.0);
            DQ_HIP(launch_splitk_reduce(gs, splits, stride, L.ld, n, n, 1.f, 0.f, G, ldg, s));
        }
    }
    return DQ_OK;
}

// ---------------------------------------------------------------- S6 (+ S7 when Zupd != null)
// What S6 needs of R and U alone, on stream s: the inverses of the diagonal blocks of U (128 x 128, merged to 512 x 512
// where the solve works on such blocks) and, for the products on three-plane splits, the planes of R (transposed for
// R^T G in x3a, as stored for R M in x3c).  (Run on the second stream beside S3-S5 it gained nothing, 8.83 ms per step
// either way at n = 4096 and 45.8 -> 46.2 at 8192: the split passes and small products land on compute units whose one
// 256 x 256 tile of the bf16 product then finishes last.  The batched 128 x 128 route does run its inverses there.)
bool backward_uses_splits(const dq_ctx* c, const Layout& L, int n) {
    return c->split_gemm != 0 && gemm_bf16x3_fits(n, n, n) && L.ld == n && (c->split_gemm == 2 || n >= 2560);
}

dq_status qr_backward_prepare(dq_ctx* c, const Layout& L, int n, const float* R, long ldr, const float* U, long ldu,
                              hipStream_t s) {
    unsigned* flags = at<unsigned>(c, L.flags);
    float* uinv = at<float>(c, L.uinv);
    const long ld = L.ld;
    const long plane = (long)n * ld;
    if (backward_uses_splits(c, L, n)) {
        LaunchScope sc(&c->prof, s, DQ_K_SMALL, 0.0, 20.0 * n * (double)n);
        DQ_HIP(launch_split3_bf16(R, ldr, n, n, at<bf16_t>(c, L.x3a), ld, plane, 1, s));
        DQ_HIP(launch_split3_bf16(R, ldr, n, n, at<bf16_t>(c, L.x3c), ld, plane, 0, s));
    }
    {
        LaunchScope sc(&c->prof, s, DQ_K_SMALL, 0.0, 8.0 * n * (double)kTrsmBlock);
        DQ_HIP(launch_trinv_blocks(U, ldu, n, uinv, flags, s));
    }
    if (n % kTrsmOuter == 0) {
        // The inverses of the 512 x 512 diagonal blocks are merged from the 128 x 128 ones, inv [[A, B], [0, C]] =
        // [[A^-1, -A^-1 B C^-1], [0, C^-1]], two levels of batched products.
        float* uo = at<float>(c, L.uinvo);
        float* t1 = at<float>(c, L.utmp);                               // n / 256 blocks of 128 x 128
        float* t2 = t1 + (size_t)n * 64;                                // n / 512 blocks of 256 x 256
        const int nouter = n / kTrsmOuter;
        const long so = (long)kTrsmOuter * kTrsmOuter;
        {
            LaunchScope sc(&c->prof, s, DQ_K_SMALL, 0.0, 4.0 * n * (double)kTrsmOuter);
            DQ_HIP(launch_place_diag_blocks(uinv, uo, n, s));
        }
        auto merge = [&](int h, int first, float* tmp, long stmp) -> dq_status {
            // for the pair of h x h diagonal blocks that starts at row `first` of every outer block:
            // tmp = B C^-1, then the upper-right block of the inverse = -A^-1 tmp
            GemmF32 g;
            g.A = U + (long)first * ldu + first + h; g.lda = ldu; g.ta = 0;
            g.B = uo + (long)(first + h) * kTrsmOuter + first + h; g.ldb = kTrsmOuter; g.tb = 0;
            g.C = tmp; g.ldc = h; g.M = h; g.N = h; g.K = h;
            g.batch = nouter; g.batch_a = (long)kTrsmOuter * ldu + kTrsmOuter; g.batch_b = so; g.batch_c = stmp;
            {
                LaunchScope sc(&c->prof, s, DQ_K_GEMM_F32, 2.0 * nouter * (double)h * h * h, 0.0);
                DQ_HIP(launch_gemm_f32(g, s));
            }
            GemmF32 f;
            f.A = uo + (long)first * kTrsmOuter + first; f.lda = kTrsmOuter; f.ta = 0;
            f.B = tmp; f.ldb = h; f.tb = 0;
            f.C = uo + (long)first * kTrsmOuter + first + h; f.ldc = kTrsmOuter; f.M = h; f.N = h; f.K = h;
            f.alpha = -1.f;
            f.batch = nouter; f.batch_a = so; f.batch_b = stmp; f.batch_c = so;
            LaunchScope sc(&c->prof, s, DQ_K_GEMM_F32, 2.0 * nouter * (double)h * h * h, 0.0);
            DQ_HIP(launch_gemm_f32(f, s));
            return DQ_OK;
        };
        DQ_TRY(merge(kTrsmBlock, 0, t1, (long)2 * kTrsmBlock * kTrsmBlock));
        DQ_TRY(merge(kTrsmBlock, 2 * kTrsmBlock, t1 + (long)kTrsmBlock * kTrsmBlock, (long)2 * kTrsmBlock * kTrsmBlock));
        DQ_TRY(merge(2 * kTrsmBlock, 0, t2, (long)4 * kTrsmBlock * kTrsmBlock));
    }
    return DQ_OK;
}

// dZ = R P U^{-T},  P = strict_lower(R^T G - G^T R).  The triangular solve M U^T = P runs right-looking over
// column blocks from the last to the first; M is strictly lower triangular, so every product skips its zero part.
// prepared: qr_backward_prepare has already run for this R and U on this stream (or the stream has waited for it).
dq_status qr_backward_one(dq_ctx* c, const Layout& L, int n, const float* R, long ldr, const float* U, long ldu,
                          const float* G, long ldg, float* dZ, long lddz, float* Zupd, long ldz, float lr,
                          bool prepared = false) {
    hipStream_t s = c->stream;
    if (!prepared) DQ_TRY(qr_backward_prepare(c, L, n, R, ldr, U, ldu, s));
    float* Bb = at<float>(c, L.B);
    float* Pb = at<float>(c, L.P);
    float* Mb = at<float>(c, L.M);
    float* uinv = at<float>(c, L.uinv);
    const long ld = L.ld;
    const double n3 = (double)n * n * n;
    // The two full n x n x n products run on the bf16 matrix cores from three-plane splits of their operands when the
    // shape fits those tiles (fp32-level accuracy: six plane pairs, fp32 accumulation), else on the fp32 ones.
    // (256 x 256 tiles at six times the matrix-core work: ahead of the fp32 kernel's 128 x 128 tiles once about a hundred of
    // them keep the compute units busy, n >= 2560)
    const bool x3 = backward_uses_splits(c, L, n);
    bf16_t* pa3 = at<bf16_t>(c, L.x3a);   // planes of R^T (qr_backward_prepare)
    bf16_t* pb3 = at<bf16_t>(c, L.x3b);   // planes of G^T, later of M
    bf16_t* pr3 = at<bf16_t>(c, L.x3c);   // planes of R (qr_backward_prepare)
    const long plane = (long)n * ld;
    if (x3) {
        {
            LaunchScope sc(&c->prof, s, DQ_K_SMALL, 0.0, 10.0 * n * (double)n);
            DQ_HIP(launch_split3_bf16(G, ldg, n, n, pb3, ld, plane, 1, s));
        }
        GemmBf16 g;   // B = R^T G:  B(i, j) = sum_k R^T(i, k) G^T(j, k)
        g.A = pa3; g.lda = ld; g.a_plane = plane;
        g.B = pb3; g.ldb = ld; g.b_plane = plane; g.tb = 1;
        g.C = Bb; g.ldc = ld; g.M = n; g.N = n; g.K = n;
        LaunchScope sc(&c->prof, s, DQ_K_GEMM_BF16, 12.0 * n3, 0.0);
        DQ_HIP(launch_gemm_bf16x3(g, s));
    } else {
        GemmF32 g;
        g.A = R; g.lda = ldr; g.ta = 1;
        g.B = G; g.ldb = ldg; g.tb = 0;
        g.C = Bb; g.ldc = ld; g.M = n; g.N = n; g.K = n;
        LaunchScope sc(&c->prof, s, DQ_K_GEMM_F32, 2.0 * n3, 0.0);
        DQ_HIP(launch_gemm_f32(g, s));
    }
    {
        LaunchScope sc(&c->prof, s, DQ_K_SMALL, 0.0, 16.0 * n * (double)n);
        DQ_HIP(launch_skew_lower(Bb, ld, n, Pb, ld, Mb, ld, s));
    }
    const int nblk = (n + kTrsmBlock - 1) / kTrsmBlock;
    if (n % kTrsmOuter == 0) {
        // M U^T = P by block columns of kTrsmOuter from the right:  M_J = P_J inv(U_JJ)^T, then everything left of the
        // block gets ONE update with K = kTrsmOuter (K = 128 updates over the whole width move P at the rate of the
        // rank-64 updates of the QR, and a chain of 128-column solves is a chain of short launches).  The inverses of
        // the 512 x 512 diagonal blocks are merged from the 128 x 128 ones, inv [[A, B], [0, C]] = [[A^-1, -A^-1 B C^-1],
        // [0, C^-1]], two levels of batched products that depend on U only.
        float* uo = at<float>(c, L.uinvo);
        const int nouter = n / kTrsmOuter;
        const long so = (long)kTrsmOuter * kTrsmOuter;
        for (int J = nouter - 1; J >= 0; --J) {
            const int J0 = J * kTrsmOuter;
            const int mrows = n - J0;
            {
                GemmF32 g;   // M[J0:, blk] = P[J0:, blk] * inv(U_JJ)^T
                g.A = Pb + (long)J0 * ld + J0; g.lda = ld; g.ta = 0;
                g.B = uo + (long)J * so; g.ldb = kTrsmOuter; g.tb = 1;
                g.C = Mb + (long)J0 * ld + J0; g.ldc = ld;
                g.M = mrows; g.N = kTrsmOuter; g.K = kTrsmOuter;
                LaunchScope sc(&c->prof, s, DQ_K_GEMM_F32, 2.0 * mrows * (double)kTrsmOuter * kTrsmOuter, 0.0);
                DQ_HIP(launch_gemm_f32(g, s));
            }
            if (J0 > 0) {
                GemmF32 g;   // P[J0:, 0:J0] -= M[J0:, blk] * U[0:J0, blk]^T (in fp32: from three-plane splits its tiles
                             // fill the compute units too unevenly to gain, 8192: 12.1 against 11.5 ms for the whole call)
                g.A = Mb + (long)J0 * ld + J0; g.lda = ld; g.ta = 0;
                g.B = U + J0; g.ldb = ldu; g.tb = 1;
                g.C = Pb + (long)J0 * ld; g.ldc = ld;
                g.M = mrows; g.N = J0; g.K = kTrsmOuter;
                g.alpha = -1.f; g.beta = 1.f;
                LaunchScope sc(&c->prof, s, DQ_K_GEMM_F32, 2.0 * mrows * (double)J0 * kTrsmOuter, 0.0);
                DQ_HIP(launch_gemm_f32(g, s));
            }
        }
    } else
    for (int j = nblk - 1; j >= 0; --j) {
        const int j0 = j * kTrsmBlock;
        const int w = (n - j0) < kTrsmBlock ? (n - j0) : kTrsmBlock;
        const int mrows = n - j0;
        {
            GemmF32 g;   // M[j0:, blk] = P[j0:, blk] * inv(U_jj)^T
            g.A = Pb + (long)j0 * ld + j0; g.lda = ld; g.ta = 0;
            g.B = uinv + (long)j * kTrsmBlock * kTrsmBlock; g.ldb = kTrsmBlock; g.tb = 1;
            g.C = Mb + (long)j0 * ld + j0; g.ldc = ld;
            g.M = mrows; g.N = w; g.K = w;
            LaunchScope sc(&c->prof, s, DQ_K_GEMM_F32, 2.0 * mrows * (double)w * w, 0.0);
            DQ_HIP(launch_gemm_f32(g, s));
        }
        if (j0 > 0) {
            GemmF32 g;   // P[j0:, 0:j0] -= M[j0:, blk] * U[0:j0, blk]^T
            g.A = Mb + (long)j0 * ld + j0; g.lda = ld; g.ta = 0;
            g.B = U + j0; g.ldb = ldu; g.tb = 1;
            g.C = Pb + (long)j0 * ld; g.ldc = ld;
            g.M = mrows; g.N = j0; g.K = w;
            g.alpha = -1.f; g.beta = 1.f;
            LaunchScope sc(&c->prof, s, DQ_K_GEMM_F32, 2.0 * mrows * (double)j0 * w, 0.0);
            DQ_HIP(launch_gemm_f32(g, s));
        }
    }
    if (x3) {
        {
            LaunchScope sc(&c->prof, s, DQ_K_SMALL, 0.0, 10.0 * n * (double)n);
            DQ_HIP(launch_split3_bf16(Mb, ld, n, n, pb3, ld, plane, 1, s));
        }
        GemmBf16 g;   // dZ = R M (or Z <- Z - lr R M):  dZ(i, j) = sum_k R(i, k) M^T(j, k), M strictly lower
        g.A = pr3; g.lda = ld; g.a_plane = plane;
        g.B = pb3; g.ldb = ld; g.b_plane = plane; g.tb = 1; g.b_strict_lower = 1;
        g.M = n; g.N = n; g.K = n;
        const int tiles = (n / 256) * (n / 256);
        if (tiles <= 256) {
            // At most one workgroup per compute unit: the triangular product in two halves of every tile's reduction range, into
            // the two n x n buffers that the solve has left free, summed by the kernel that also applies the step.  Whole,
            // the longest tile alone takes as long as the full product (n = 4096: 632 -> 361 + 42 us; with 400 tiles,
            // n = 5120, dealing the tiles out longest first already balances them: 3.50 -> 3.56 ms for the whole call).
            g.C = Bb; g.ldc = ld; g.splits = 2; g.split_stride = Pb - Bb;
            {
                LaunchScope sc(&c->prof, s, DQ_K_GEMM_BF16, 6.0 * n3, 0.0);
                DQ_HIP(launch_gemm_bf16x3(g, s));
            }
            LaunchScope sc(&c->prof, s, DQ_K_SMALL, 0.0, 16.0 * n * (double)n);
            if (Zupd != nullptr) DQ_HIP(launch_splitk_reduce(Bb, 2, Pb - Bb, ld, n, n, -lr, 1.f, Zupd, ldz, s));
            else DQ_HIP(launch_splitk_reduce(Bb, 2, Pb - Bb, ld, n, n, 1.f, 0.f, dZ, lddz, s));
            return DQ_OK;
        }
        if (Zupd != nullptr) { g.C = Zupd; g.ldc = ldz; g.alpha = -lr; g.beta = 1.f; }
        else { g.C = dZ; g.ldc = lddz; }
        LaunchScope sc(&c->prof, s, DQ_K_GEMM_BF16, 6.0 * n3, 0.0);
        DQ_HIP(launch_gemm_bf16x3(g, s));
    } else {
        GemmF32 g;   // dZ = R * M  (or Z <- Z - lr * R * M)
        g.A = R; g.lda = ldr; g.ta = 0;
        g.B = Mb; g.ldb = ld; g.tb = 0; g.b_strict_lower = 1;
        g.M = n; g.N = n; g.K = n;
        if (Zupd != nullptr) { g.C = Zupd; g.ldc = ldz; g.alpha = -lr; g.beta = 1.f; }
        else { g.C = dZ; g.ldc = lddz; }
        LaunchScope sc(&c->prof, s, DQ_K_GEMM_F32, n3, 0.0);
        DQ_HIP(launch_gemm_f32(g, s));
    }
    return DQ_OK;
}

// ---------------------------------------------------------------- Cayley SGD with momentum (Alg. 3, App. B.2)
// One update of the rotation R (the algorithm's X_k) from its Euclidean gradient G, in the algorithm's own order:
//   M <- beta M - G;  W^ = M R^T - 1/2 R (R^T M R^T);  W = W^ - W^^T;  M <- W R;  alpha = min(lr, 2q / (||W||_F + eps));
//   Y = R + alpha M;  s times: Y <- R + alpha/2 W (R + Y);  R <- Y.
// Six n x n products on the fp32 matrix cores; the step size stays on the device.
dq_status cayley_update_one(dq_ctx* c, const Layout& L, int n, float* R, long ldr, const float* G, long ldg, float* M,
                            long ldm, float lr, float beta, float q, int iters, float eps, float* alpha_out) {
    hipStream_t s = c->stream;
    const long ld = L.ld;
    float* What = at<float>(c, L.B);     // A = M R^T, then W^
    float* Tmp = at<float>(c, L.P);      // R^T A, later R + Y
    float* W = at<float>(c, L.M);
    float* Y0 = at<float>(c, L.U);
    float* Y1 = at<float>(c, L.A);
    double* part = at<double>(c, L.losspart);
    float* scal = at<float>(c, L.scal);
    const double n3 = (double)n * n * n;
    // As in S6, the products run on the bf16 matrix cores from three-plane splits when the shape fits (DQ_OPT_SPLIT_GEMM):
    // `pa` holds the planes of op(A) (n x n, reduction index contiguous), `pb` those of op(B)^T; a null `A_` / `B_` means
    // that the buffer already holds them from an earlier product.
    const bool x3 = c->split_gemm != 0 && gemm_bf16x3_fits(n, n, n) && ld == n && (c->split_gemm == 2 || n >= 2560);
    const long plane = (long)n * ld;
    bf16_t* pl0 = at<bf16_t>(c, L.x3a);
    bf16_t* pl1 = at<bf16_t>(c, L.x3b);
    bf16_t* pl2 = at<bf16_t>(c, L.x3c);
    bf16_t* pl3 = at<bf16_t>(c, L.x3d);
    auto product = [&](const float* A_, long lda, int ta, bf16_t* pa, const float* B_, long ldb, int tb, bf16_t* pb,
                       float* C_, long ldc, float alpha, float beta_, const float* alpha_dev) -> dq_status {
        if (x3) {
            {
                LaunchScope sc(&c->prof, s, DQ_K_SMALL, 0.0, 10.0 * n * (double)n);
                if (A_ != nullptr) DQ_HIP(launch_split3_bf16(A_, lda, n, n, pa, ld, plane, ta ? 1 : 0, s));
                if (B_ != nullptr) DQ_HIP(launch_split3_bf16(B_, ldb, n, n, pb, ld, plane, tb ? 0 : 1, s));
            }
            GemmBf16 g;
            g.A = pa; g.lda = ld; g.a_plane = plane;
            g.B = pb; g.ldb = ld; g.b_plane = plane; g.tb = 1;
            g.C = C_; g.ldc = ldc; g.M = n; g.N = n; g.K = n;
            g.alpha = alpha; g.beta = beta_; g.alpha_dev = alpha_dev;
            LaunchScope sc(&c->prof, s, DQ_K_GEMM_BF16, 12.0 * n3, 0.0);
            DQ_HIP(launch_gemm_bf16x3(g, s));
            return DQ_OK;
        }
        if (A_ == nullptr || B_ == nullptr) return DQ_ERR_NULL;
        GemmF32 g;
        g.A = A_; g.lda = lda; g.ta = ta;
        g.B = B_; g.ldb = ldb; g.tb = tb;
        g.C = C_; g.ldc = ldc; g.M = n; g.N = n; g.K = n;
        g.alpha = alpha; g.beta = beta_; g.alpha_dev = alpha_dev;
        LaunchScope sc(&c->prof, s, DQ_K_GEMM_F32, 2.0 * n3, 0.0);
        DQ_HIP(launch_gemm_f32(g, s));
        return DQ_OK;
    };
    {
        LaunchScope sc(&c->prof, s, DQ_K_SMALL, 2.0 * n * (double)n, 12.0 * n * (double)n);
        DQ_HIP(launch_cayley_momentum(M, ldm, G, ldg, n, beta, s));
    }
    DQ_TRY(product(M, ldm, 0, pl0, R, ldr, 1, pl1, What, ld, 1.f, 0.f, nullptr));          // A = M R^T
    DQ_TRY(product(R, ldr, 1, pl2, What, ld, 0, pl0, Tmp, ld, 1.f, 0.f, nullptr));         // R^T A
    // (x3: the planes of R are in pl1 since the first product, those of R^T stay in pl2 for the fourth)
    DQ_TRY(product(x3 ? nullptr : R, ldr, 0, pl1, Tmp, ld, 0, pl0, What, ld, -0.5f, 1.f, nullptr));       // W^ = A - 1/2 R (R^T A)
    const int blocks = cayley_skew_grid(n);
    if (blocks > kLossPartials) return DQ_ERR_UNSUPPORTED;
    {
        LaunchScope sc(&c->prof, s, DQ_K_SMALL, 3.0 * n * (double)n, 12.0 * n * (double)n);
        DQ_HIP(launch_cayley_skew(What, ld, n, W, ld, part, s));
        DQ_HIP(launch_cayley_alpha(part, blocks, lr, q, eps, scal, s));
    }
    DQ_TRY(product(W, ld, 0, pl3, x3 ? nullptr : R, ldr, 0, pl2, M, ldm, 1.f, 0.f, nullptr));             // M = W R
    {
        LaunchScope sc(&c->prof, s, DQ_K_SMALL, 2.0 * n * (double)n, 12.0 * n * (double)n);
        DQ_HIP(launch_add_scaled(Y0, ld, R, ldr, M, ldm, n, 1.f, scal, s));      // Y = R + alpha M
    }
    float* Ycur = Y0;
    float* Ynext = Y1;
    for (int i = 0; i < iters; ++i) {
        {
            LaunchScope sc(&c->prof, s, DQ_K_SMALL, 1.0 * n * (double)n, 20.0 * n * (double)n);
            DQ_HIP(launch_add_scaled(Tmp, ld, R, ldr, Ycur, ld, n, 1.f, nullptr, s));   // R + Y
            DQ_HIP(launch_copy2d(R, ldr, Ynext, ld, n, n, s));
        }
        DQ_TRY(product(x3 ? nullptr : W, ld, 0, pl3, Tmp, ld, 0, pl0, Ynext, ld, 1.f, 1.f, scal + 1));    // Y <- R + alpha/2 W (R + Y)
        float* t = Ycur; Ycur = Ynext; Ynext = t;
    }
    {
        LaunchScope sc(&c->prof, s, DQ_K_SMALL, 0.0, 8.0 * n * (double)n);
        DQ_HIP(launch_copy2d(Ycur, ld, R, ldr, n, n, s));
        if (alpha_out != nullptr) DQ_HIP(launch_copy2d(scal, 4, alpha_out, 4, 1, 1, s));
    }
    return DQ_OK;
}

// ---------------------------------------------------------------- batched 128 x 128 rotations
// Every problem of the batch runs in the same launches.  The path's buffers (b matrices each, row stride 128) sit
// behind the general layout in the workspace.
struct HeadsLayout {
    size_t R = 0, U = 0, G = 0, B = 0, P = 0, M = 0, uinv = 0, gpart = 0, lpart = 0, total = 0;
};

HeadsLayout make_heads_layout(size_t base, int b, int T) {
    HeadsLayout H;
    size_t cur = base;
    const size_t mat = (size_t)(b > 0 ? b : 1) * kHeadDim * kHeadDim * 4;
    const size_t sp = (size_t)heads_splits(T > 0 ? T : 1);
    H.R = bump(cur, mat);
    H.U = bump(cur, mat);
    H.G = bump(cur, mat);
    H.B = bump(cur, mat);
    H.P = bump(cur, mat);
    H.M = bump(cur, mat);
    H.uinv = bump(cur, mat);
    H.gpart = bump(cur, mat * sp);
    H.lpart = bump(cur, (size_t)(b > 0 ? b : 1) * sp * 8);
    H.total = cur;
    return H;
}

bool heads_route(const dq_ctx* c, int n) { return c->heads_batched && n == kHeadDim; }
// the fused rotate + loss + gradient kernel of the batched route evaluates Eq. 4 only
bool heads_fused_route(const dq_ctx* c, int n) { return heads_route(c, n) && c->objective == DQ_OBJ_WHIP; }

dq_status check_heads_ws(dq_ctx* c, const HeadsLayout& H) {
    if (c->ws == nullptr || c->ws_bytes < H.total) return DQ_ERR_WORKSPACE;
    return DQ_OK;
}

dq_status heads_qr(dq_ctx* c, int b, const float* Z, long ldz, float* R, long ldr, float* U, long ldu) {
    const int n = kHeadDim;
    if (b < 1) return DQ_OK;
    LaunchScope sc(&c->prof, c->stream, DQ_K_PANEL, b * (10.0 / 3.0) * n * (double)n * n, 0.0);
    DQ_HIP(launch_heads_qr(b, Z, ldz, (long)n * ldz, R, ldr, (long)n * ldr, U, ldu, (long)n * ldu,
                           at<unsigned>(c, 0), c->stream));
    return DQ_OK;
}

dq_status heads_rotate_loss_grad(dq_ctx* c, const HeadsLayout& H, int b, int T, const void* X, long ldx, const float* R,
                                 long ldr, dq_reduce red, float* loss_dev, float* G, long ldg) {
    const int n = kHeadDim;
    if (b < 1) return DQ_OK;
    const float scale = (red == DQ_REDUCE_TOKEN_MEAN) ? 1.f / (float)T : 1.f;
    LaunchScope sc(&c->prof, c->stream, DQ_K_GEMM_BF16, b * 4.0 * T * (double)n * n, b * 2.0 * T * (double)n);
    DQ_HIP(launch_heads_rlg(b, T, static_cast<const bf16_t*>(X), ldx, (long)T * ldx, R, ldr, (long)n * ldr, scale,
                            at<float>(c, H.gpart), at<double>(c, H.lpart), G, ldg, (long)n * ldg, loss_dev,
                            at<unsigned>(c, 0), c->stream));
    return DQ_OK;
}

// inv(U_i) for every problem on the second stream, beside whatever the caller's stream does next: it depends on the
// factorisation only, and the 64 workgroups that form it (a quarter of the device, 30 us) need not sit between the
// gradient and the derivative through the QR.  The caller's stream must wait for sync_ev[1] before inv(U) is used.
dq_status heads_uinv_early(dq_ctx* c, const HeadsLayout& H, int b, const float* U, long ldu) {
    const int n = kHeadDim;
    DQ_HIP(hipEventRecord(c->sync_ev[0], c->stream));
    DQ_HIP(hipStreamWaitEvent(c->stream2, c->sync_ev[0], 0));
    {
        LaunchScope sc(&c->prof, c->stream2, DQ_K_SMALL, 0.0, 8.0 * b * (double)n * n);
        DQ_HIP(launch_trinv_blocks(U, ldu, n, at<float>(c, H.uinv), at<unsigned>(c, 0), c->stream2, b, (long)n * ldu,
                                   (long)n * n));
    }
    DQ_HIP(hipEventRecord(c->sync_ev[1], c->stream2));
    return DQ_OK;
}

// dZ_i = R_i P_i U_i^{-T} for every problem (or Z_i -= lr dZ_i when Zupd != null): the steps of qr_backward_one with
// one 128-wide block, as batched launches.  have_uinv: inv(U_i) is already in the workspace (heads_uinv_early).
dq_status heads_backward(dq_ctx* c, const HeadsLayout& H, int b, const float* R, long ldr, const float* U, long ldu,
                         const float* G, long ldg, float* dZ, long lddz, float* Zupd, long ldz, float lr,
                         bool have_uinv = false) {
    const int n = kHeadDim;
    const long nn = (long)n * n;
    if (b < 1) return DQ_OK;
    hipStream_t s = c->stream;
    unsigned* flags = at<unsigned>(c, 0);
    float* Bb = at<float>(c, H.B);
    float* Pb = at<float>(c, H.P);
    float* Mb = at<float>(c, H.M);
    float* uinv = at<float>(c, H.uinv);
    const double n3 = (double)b * n * n * n;
    {
        GemmF32 g;   // B = R^T G
        g.A = R; g.lda = ldr; g.ta = 1; g.batch_a = (long)n * ldr;
        g.B = G; g.ldb = ldg; g.tb = 0; g.batch_b = (long)n * ldg;
        g.C = Bb; g.ldc = n; g.batch_c = nn;
        g.M = n; g.N = n; g.K = n; g.batch = b;
        LaunchScope sc(&c->prof, s, DQ_K_GEMM_F32, 2.0 * n3, 0.0);
        DQ_HIP(launch_gemm_f32(g, s));
    }
    {
        LaunchScope sc(&c->prof, s, DQ_K_SMALL, 0.0, 16.0 * b * (double)nn);
        DQ_HIP(launch_skew_lower(Bb, n, n, Pb, n, nullptr, 0, s, b, nn, nn, 0));
        if (!have_uinv) DQ_HIP(launch_trinv_blocks(U, ldu, n, uinv, flags, s, b, (long)n * ldu, nn));
    }
    {
        GemmF32 g;   // M = P inv(U)^T
        g.A = Pb; g.lda = n; g.ta = 0; g.batch_a = nn;
        g.B = uinv; g.ldb = kTrsmBlock; g.tb = 1; g.batch_b = nn;
        g.C = Mb; g.ldc = n; g.batch_c = nn;
        g.M = n; g.N = n; g.K = n; g.batch = b;
        LaunchScope sc(&c->prof, s, DQ_K_GEMM_F32, 2.0 * n3, 0.0);
        DQ_HIP(launch_gemm_f32(g, s));
    }
    {
        GemmF32 g;   // dZ = R M  (or Z <- Z - lr R M)
        g.A = R; g.lda = ldr; g.ta = 0; g.batch_a = (long)n * ldr;
        g.B = Mb; g.ldb = n; g.tb = 0; g.b_strict_lower = 1; g.batch_b = nn;
        g.M = n; g.N = n; g.K = n; g.batch = b;
        if (Zupd != nullptr) { g.C = Zupd; g.ldc = ldz; g.batch_c = (long)n * ldz; g.alpha = -lr; g.beta = 1.f; }
        else { g.C = dZ; g.ldc = lddz; g.batch_c = (long)n * lddz; }
        LaunchScope sc(&c->prof, s, DQ_K_GEMM_F32, n3, 0.0);
        DQ_HIP(launch_gemm_f32(g, s));
    }
    return DQ_OK;
}

}  // namespace

// =================================================================== C ABI
extern "C" {

const char* dq_status_string(dq_status s) {
    switch (s) {
        case DQ_OK: return "ok";
        case DQ_ERR_NULL: return "null pointer";
        case DQ_ERR_SHAPE: return "bad shape or leading dimension";
        case DQ_ERR_DTYPE: return "bad dtype or reduce mode";
        case DQ_ERR_ALIGN: return "pointer or leading dimension misaligned";
        case DQ_ERR_WORKSPACE: return "workspace missing or too small";
        case DQ_ERR_HIP: return "HIP runtime error";
        case DQ_ERR_UNSUPPORTED: return "size outside the supported range";
    }
    return "unknown status";
}

dq_status dq_create(dq_ctx** out, void* hip_stream) {
    if (out == nullptr) return DQ_ERR_NULL;
    dq_ctx* c = new (std::nothrow) dq_ctx();
    if (c == nullptr) return DQ_ERR_HIP;
    c->stream = static_cast<hipStream_t>(hip_stream);
    // a context that cannot be created says why on stderr: there is no other channel yet
    auto fail = [&](const char* what, hipError_t e) {
        fprintf(stderr, "dq_create: %s failed: %s\n", what, hipGetErrorString(e));
        dq_destroy(c);
        return DQ_ERR_HIP;
    };
    hipError_t e = hipGetDevice(&c->device);
    if (e != hipSuccess) return fail("hipGetDevice", e);
    // default priority on purpose; non-blocking so that they never synchronise with the legacy default stream
    hipStream_t* internal[3] = {&c->stream2, &c->stream3, nullptr};
    for (int i = 0; internal[i] != nullptr; ++i)
        if ((e = hipStreamCreateWithFlags(internal[i], hipStreamNonBlocking)) != hipSuccess)
            return fail("hipStreamCreateWithFlags", e);
    const int nev = 2 * (DQ_MAX_N / kPanel) + 1;
    for (int i = 0; i < nev; ++i) {
        hipEvent_t ev;
        // These events order kernels on streams of this device only: no timing, and no system-scope fence (the cache
        // write-back that makes device memory visible to the host and to other devices) when one is recorded.
        if ((e = hipEventCreateWithFlags(&ev, hipEventDisableTiming | hipEventDisableSystemFence)) != hipSuccess)
            return fail("hipEventCreateWithFlags", e);
        c->sync_ev.push_back(ev);
    }
    *out = c;
    return DQ_OK;
}

dq_status dq_destroy(dq_ctx* c) {
    if (c == nullptr) return DQ_ERR_NULL;
    if (c->stream2 != nullptr) (void)hipStreamSynchronize(c->stream);   // a context that got as far as launching
    if (c->stream2 != nullptr) { (void)hipStreamSynchronize(c->stream2); (void)hipStreamDestroy(c->stream2); }
    if (c->stream3 != nullptr) { (void)hipStreamSynchronize(c->stream3); (void)hipStreamDestroy(c->stream3); }
    if (c->copy_stream != nullptr) { (void)hipStreamSynchronize(c->copy_stream); (void)hipStreamDestroy(c->copy_stream); }
    for (int i = 0; i < 2; ++i) {
        if (c->batch_ready[i] != nullptr) (void)hipEventDestroy(c->batch_ready[i]);
        if (c->batch_done[i] != nullptr) (void)hipEventDestroy(c->batch_done[i]);
    }
    for (hipEvent_t e : c->prof.ev) (void)hipEventDestroy(e);
    for (hipEvent_t e : c->sync_ev) (void)hipEventDestroy(e);
    delete c;
    return DQ_OK;
}

dq_status dq_workspace_bytes(int b, int n, int T, dq_dtype x_dtype, size_t* out) {
    if (out == nullptr) return DQ_ERR_NULL;
    if (b < 0 || T < 1) return DQ_ERR_SHAPE;
    DQ_TRY(check_n(n));
    if (x_dtype != DQ_F32 && x_dtype != DQ_BF16) return DQ_ERR_DTYPE;
    const Layout L = make_layout(n, T);
    *out = n == kHeadDim ? make_heads_layout(L.total, b, T).total : L.total;
    return DQ_OK;
}

dq_status dq_set_workspace(dq_ctx* c, void* dptr, size_t bytes) {
    if (c == nullptr || dptr == nullptr) return DQ_ERR_NULL;
    if ((reinterpret_cast<uintptr_t>(dptr) & 255) != 0) return DQ_ERR_ALIGN;
    if (bytes < 256) return DQ_ERR_WORKSPACE;
    c->ws = static_cast<char*>(dptr);
    c->ws_bytes = bytes;
    DQ_HIP(launch_fill_u32(reinterpret_cast<unsigned*>(c->ws), 64, 0u, c->stream));
    c->arrived = 0;
    c->arrived_rows = 0;
    return DQ_OK;
}

dq_status dq_device_flags(dq_ctx* c, unsigned* host_out) {
    if (c == nullptr || host_out == nullptr) return DQ_ERR_NULL;
    if (c->ws == nullptr) return DQ_ERR_WORKSPACE;
    DQ_HIP(hipMemcpyAsync(host_out, c->ws, sizeof(unsigned), hipMemcpyDeviceToHost, c->stream));
    DQ_HIP(hipStreamSynchronize(c->stream));
    DQ_HIP(launch_fill_u32(reinterpret_cast<unsigned*>(c->ws), 64, 0u, c->stream));
    c->arrived = 0;
    c->arrived_rows = 0;
    return DQ_OK;
}

dq_status dq_qr_orth(dq_ctx* c, int b, int n, const float* Z, long ldz, float* R, long ldr, float* U, long ldu) {
    if (c == nullptr) return DQ_ERR_NULL;
    if (b < 0) return DQ_ERR_SHAPE;
    DQ_TRY(check_n(n));
    DQ_TRY(check_f32(Z, ldz, n));
    DQ_TRY(check_f32(R, ldr, n));
    if (U != nullptr) DQ_TRY(check_f32(U, ldu, n));
    const Layout L = make_layout(n, 1);
    DQ_TRY(check_ws(c, L));
    if (heads_route(c, n)) return heads_qr(c, b, Z, ldz, R, ldr, U, ldu);
    for (int i = 0; i < b; ++i)
        DQ_TRY(qr_orth_one(c, L, n, Z + (long)i * n * ldz, ldz, R + (long)i * n * ldr, ldr,
                           U ? U + (long)i * n * ldu : nullptr, ldu));
    return DQ_OK;
}

dq_status dq_rotate_loss_grad(dq_ctx* c, int b, int T, int n, const void* X, dq_dtype xdt, long ldx, const float* R,
                              long ldr, dq_reduce red, float* loss_dev, float* G, long ldg, float* Y, long ldy,
                              void* dY, long lddy) {
    if (c == nullptr || loss_dev == nullptr) return DQ_ERR_NULL;
    if (b < 0 || T < 1) return DQ_ERR_SHAPE;
    DQ_TRY(check_n(n));
    if (red != DQ_REDUCE_TOKEN_MEAN && red != DQ_REDUCE_SUM) return DQ_ERR_DTYPE;
    DQ_TRY(check_x(X, xdt, ldx, n));
    DQ_TRY(check_f32(R, ldr, n));
    DQ_TRY(check_f32(G, ldg, n));
    if (Y != nullptr) DQ_TRY(check_f32(Y, ldy, n));
    if (dY != nullptr) DQ_TRY(check_x(dY, xdt, lddy, n));
    const Layout L = make_layout(n, T);
    DQ_TRY(check_ws(c, L));
    if (heads_fused_route(c, n) && xdt == DQ_BF16 && Y == nullptr && dY == nullptr) {
        const HeadsLayout H = make_heads_layout(L.total, b, T);
        DQ_TRY(check_heads_ws(c, H));
        return heads_rotate_loss_grad(c, H, b, T, X, ldx, R, ldr, red, loss_dev, G, ldg);
    }
    const size_t esz = (xdt == DQ_BF16) ? 2 : 4;
    for (int i = 0; i < b; ++i) {
        float* Yi = Y ? Y + (long)i * T * ldy : at<float>(c, L.Y);
        const long ldyi = Y ? ldy : L.ld;
        void* dYi = dY ? static_cast<void*>(static_cast<char*>(dY) + (size_t)i * T * lddy * esz)
                       : static_cast<void*>(at<char>(c, L.dY));
        const long lddyi = dY ? lddy : L.ld;
        const void* Xi = static_cast<const char*>(X) + (size_t)i * T * ldx * esz;
        DQ_TRY(rotate_loss_grad_one(c, L, T, n, Xi, xdt, ldx, R + (long)i * n * ldr, ldr, red, loss_dev + i,
                                    G + (long)i * n * ldg, ldg, Yi, ldyi, dYi, lddyi, Y != nullptr || dY != nullptr));
    }
    return DQ_OK;
}

dq_status dq_calib_step(dq_ctx* c, int b, int T, int n, const void* X, dq_dtype xdt, long ldx, float* Z, long ldz,
                        float lr, dq_reduce red, float* loss_dev, float* R, long ldr) {
    if (c == nullptr || loss_dev == nullptr) return DQ_ERR_NULL;
    if (b < 0 || T < 1) return DQ_ERR_SHAPE;
    DQ_TRY(check_n(n));
    if (red != DQ_REDUCE_TOKEN_MEAN && red != DQ_REDUCE_SUM) return DQ_ERR_DTYPE;
    DQ_TRY(check_x(X, xdt, ldx, n));
    DQ_TRY(check_f32(Z, ldz, n));
    if (R != nullptr) DQ_TRY(check_f32(R, ldr, n));
    const Layout L = make_layout(n, T);
    DQ_TRY(check_ws(c, L));
    if (heads_fused_route(c, n) && xdt == DQ_BF16) {
        const HeadsLayout H = make_heads_layout(L.total, b, T);
        DQ_TRY(check_heads_ws(c, H));
        float* Rh = R ? R : at<float>(c, H.R);
        const long ldrh = R ? ldr : kHeadDim;
        float* Uh = at<float>(c, H.U);
        float* Gh = at<float>(c, H.G);
        DQ_TRY(heads_qr(c, b, Z, ldz, Rh, ldrh, Uh, kHeadDim));
        const bool early = !c->single_stream && b >= 1;
        if (early) DQ_TRY(heads_uinv_early(c, H, b, Uh, kHeadDim));
        DQ_TRY(heads_rotate_loss_grad(c, H, b, T, X, ldx, Rh, ldrh, red, loss_dev, Gh, kHeadDim));
        if (early) DQ_HIP(hipStreamWaitEvent(c->stream, c->sync_ev[1], 0));
        return heads_backward(c, H, b, Rh, ldrh, Uh, kHeadDim, Gh, kHeadDim, nullptr, 0, Z, ldz, lr, early);
    }
    const size_t esz = (xdt == DQ_BF16) ? 2 : 4;
    for (int i = 0; i < b; ++i) {
        float* Zi = Z + (long)i * n * ldz;
        float* Ri = R ? R + (long)i * n * ldr : at<float>(c, L.R);
        const long ldri = R ? ldr : L.ld;
        // The rotation is sign-normalised whether or not it is reported.  Loss and dL/dZ do not depend on the column
        // signs in exact arithmetic, but the bf16 matrix cores do not round sign-symmetrically, and dY is discontinuous
        // at y = 0: a step on R S would differ from the staged calls (which see the normalised R) by the entries of Y
        // at rounding level.  One pass over three n x n matrices keeps the two routes identical.
        float* Ui = at<float>(c, L.U);
        float* Gi = at<float>(c, L.G);
        const void* Xi = static_cast<const char*>(X) + (size_t)i * T * ldx * esz;
        DQ_TRY(qr_orth_one(c, L, n, Zi, ldz, Ri, ldri, Ui, L.ld));
        DQ_TRY(rotate_loss_grad_one(c, L, T, n, Xi, xdt, ldx, Ri, ldri, red, loss_dev + i, Gi, L.ld,
                                    at<float>(c, L.Y), L.ld, at<char>(c, L.dY), L.ld, false));
        DQ_TRY(qr_backward_one(c, L, n, Ri, ldri, Ui, L.ld, Gi, L.ld, nullptr, 0, Zi, ldz, lr));
    }
    return DQ_OK;
}

dq_status dq_calib_run_host_batches(dq_ctx* c, int T, int n, const void* const* X_host, int num_batches, dq_dtype xdt,
                                    long ldx, void* staging_dev, float* Z, long ldz, float lr, dq_reduce red, int steps,
                                    float* losses_dev) {
    if (c == nullptr || X_host == nullptr || staging_dev == nullptr || Z == nullptr || losses_dev == nullptr)
        return DQ_ERR_NULL;
    if (T < 1 || num_batches < 1 || steps < 0) return DQ_ERR_SHAPE;
    DQ_TRY(check_n(n));
    DQ_TRY(check_x(staging_dev, xdt, ldx, n));
    DQ_TRY(check_f32(Z, ldz, n));
    if (red != DQ_REDUCE_TOKEN_MEAN && red != DQ_REDUCE_SUM) return DQ_ERR_DTYPE;
    for (int i = 0; i < num_batches; ++i)
        if (X_host[i] == nullptr) return DQ_ERR_NULL;
    size_t need = 0;
    DQ_TRY(dq_workspace_bytes(1, n, T, xdt, &need));
    if (c->ws == nullptr || c->ws_bytes < need) return DQ_ERR_WORKSPACE;
    if (steps == 0) return DQ_OK;
    if (c->copy_stream == nullptr) {
        // default priority, like every stream of this library
        if (hipStreamCreateWithFlags(&c->copy_stream, hipStreamNonBlocking) != hipSuccess) return DQ_ERR_HIP;
        for (int i = 0; i < 2; ++i) {
            DQ_HIP(hipEventCreateWithFlags(&c->batch_ready[i], hipEventDisableTiming));
            DQ_HIP(hipEventCreateWithFlags(&c->batch_done[i], hipEventDisableTiming));
        }
    }
    const size_t esz = (xdt == DQ_BF16) ? 2 : 4;
    const size_t batch_bytes = (size_t)T * ldx * esz;
    char* slot[2] = {static_cast<char*>(staging_dev), static_cast<char*>(staging_dev) + batch_bytes};
    // whatever the caller's stream still does with the staging memory comes first
    DQ_HIP(hipEventRecord(c->batch_done[0], c->stream));
    DQ_HIP(hipStreamWaitEvent(c->copy_stream, c->batch_done[0], 0));
    DQ_HIP(hipMemcpyAsync(slot[0], X_host[0], batch_bytes, hipMemcpyHostToDevice, c->copy_stream));
    DQ_HIP(hipEventRecord(c->batch_ready[0], c->copy_stream));
    for (int k = 0; k < steps; ++k) {
        const int cur = k & 1, nxt = cur ^ 1;
        if (k + 1 < steps) {
            // the other slot was last read by step k - 1
            if (k >= 1) DQ_HIP(hipStreamWaitEvent(c->copy_stream, c->batch_done[nxt], 0));
            DQ_HIP(hipMemcpyAsync(slot[nxt], X_host[(k + 1) % num_batches], batch_bytes, hipMemcpyHostToDevice,
                                  c->copy_stream));
            DQ_HIP(hipEventRecord(c->batch_ready[nxt], c->copy_stream));
        }
        DQ_HIP(hipStreamWaitEvent(c->stream, c->batch_ready[cur], 0));
        DQ_TRY(dq_calib_step(c, 1, T, n, slot[cur], xdt, ldx, Z, ldz, lr, red, losses_dev + k, nullptr, 0));
        DQ_HIP(hipEventRecord(c->batch_done[cur], c->stream));
    }
    return DQ_OK;
}

dq_status dq_whip_loss_grad(dq_ctx* c, int b, int T, int n, const float* Y, long ldy, dq_reduce red, float* loss_dev,
                            void* dY, dq_dtype dydt, long lddy) {
    if (c == nullptr || loss_dev == nullptr) return DQ_ERR_NULL;
    if (b < 0 || T < 1 || n < 1) return DQ_ERR_SHAPE;
    if (red != DQ_REDUCE_TOKEN_MEAN && red != DQ_REDUCE_SUM) return DQ_ERR_DTYPE;
    DQ_TRY(check_f32(Y, ldy, n));
    DQ_TRY(check_x(dY, dydt, lddy, n));
    if (c->ws == nullptr || c->ws_bytes < make_layout(1, 1).total) return DQ_ERR_WORKSPACE;
    // only the status word and the loss partials are needed: they sit at fixed offsets of the n = 1 layout
    const Layout L = make_layout(1, 1);
    unsigned* flags = at<unsigned>(c, L.flags);
    double* lpart = at<double>(c, L.losspart);
    const float scale = (red == DQ_REDUCE_TOKEN_MEAN) ? 1.f / (float)T : 1.f;
    const size_t esz = (dydt == DQ_BF16) ? 2 : 4;
    if (b == 0) return DQ_OK;
    // every problem of the batch in the same two launches; the partial sums of problem i sit at lpart + i * grid
    int grid = whip_grid(T, n);
    if ((long)grid * b > kLossPartials) grid = kLossPartials / b;
    if (grid < 1) return DQ_ERR_UNSUPPORTED;
    {
        LaunchScope sc(&c->prof, c->stream, DQ_K_WHIP, 5.0 * b * T * (double)n, (double)b * T * n * (4.0 + esz));
        DQ_HIP(launch_whip(Y, ldy, T, n, scale, dY, dydt == DQ_BF16, lddy, lpart, grid, c->stream, b, (long)T * ldy,
                           (long)T * lddy));
    }
    DQ_HIP(launch_loss_finish(lpart, grid, scale, loss_dev, flags, c->stream, b));
    return DQ_OK;
}

dq_status dq_whip_loss_grad_noalloc(void* hip_stream, int b, int T, int n, const float* Y, long ldy, dq_reduce red,
                                    float* loss_dev, void* dY, dq_dtype dydt, long lddy) {
    if (loss_dev == nullptr) return DQ_ERR_NULL;
    if (b < 0 || T < 1 || n < 1) return DQ_ERR_SHAPE;
    if (b > DQ_NOALLOC_MAX_BATCH) return DQ_ERR_UNSUPPORTED;
    if (red != DQ_REDUCE_TOKEN_MEAN && red != DQ_REDUCE_SUM) return DQ_ERR_DTYPE;
    DQ_TRY(check_f32(Y, ldy, n));
    DQ_TRY(check_x(dY, dydt, lddy, n));
    if (b == 0) return DQ_OK;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    void* base = nullptr;
    DQ_HIP(noalloc_scratch(&base));
    unsigned* flags = static_cast<unsigned*>(base);
    double* lpart = reinterpret_cast<double*>(static_cast<char*>(base) + 256);
    const float scale = (red == DQ_REDUCE_TOKEN_MEAN) ? 1.f / (float)T : 1.f;
    int grid = whip_grid(T, n);
    if ((long)grid * b > kNoallocPartials) grid = kNoallocPartials / b;   // >= 1 since b <= kNoallocPartials
    // the array keeps what the last call left: the status word starts from zero (a fill kernel, so that the call can
    // be recorded into a HIP graph); every partial the finish kernel reads is written by this call's Whip pass
    DQ_HIP(launch_fill_u32(flags, 64, 0u, s));
    DQ_HIP(launch_whip(Y, ldy, T, n, scale, dY, dydt == DQ_BF16, lddy, lpart, grid, s, b, (long)T * ldy, (long)T * lddy));
    DQ_HIP(launch_loss_finish(lpart, grid, scale, loss_dev, flags, s, b));
    return DQ_OK;
}

dq_status dq_objective_loss_grad(dq_ctx* c, dq_objective objective, int quant_bits, int b, int T, int n, const float* Y,
                                 long ldy, dq_reduce red, float* loss_dev, void* dY, dq_dtype dydt, long lddy) {
    if (objective == DQ_OBJ_WHIP) return dq_whip_loss_grad(c, b, T, n, Y, ldy, red, loss_dev, dY, dydt, lddy);
    if (c == nullptr || loss_dev == nullptr) return DQ_ERR_NULL;
    if (objective != DQ_OBJ_VARIANCE && objective != DQ_OBJ_KURTOSIS && objective != DQ_OBJ_QUANT) return DQ_ERR_DTYPE;
    if (b < 0 || T < 1 || n < 1 || quant_bits < 1 || quant_bits > 16) return DQ_ERR_SHAPE;
    if (n > DQ_MAX_N) return DQ_ERR_UNSUPPORTED;
    if (red != DQ_REDUCE_TOKEN_MEAN && red != DQ_REDUCE_SUM) return DQ_ERR_DTYPE;
    DQ_TRY(check_f32(Y, ldy, n));
    if (dY != nullptr) DQ_TRY(check_x(dY, dydt, lddy, n));     // no dY: the loss alone (an evaluation metric)
    else if (dydt != DQ_F32 && dydt != DQ_BF16) return DQ_ERR_DTYPE;
    if (c->ws == nullptr || c->ws_bytes < make_layout(1, 1).total) return DQ_ERR_WORKSPACE;
    const Layout L = make_layout(1, 1);
    unsigned* flags = at<unsigned>(c, L.flags);
    double* lpart = at<double>(c, L.losspart);
    const float scale = (red == DQ_REDUCE_TOKEN_MEAN) ? 1.f / (float)T : 1.f;
    const size_t esz = dY == nullptr ? 0 : ((dydt == DQ_BF16) ? 2 : 4);
    if (b == 0) return DQ_OK;
    int grid = objective_grid(T, n);
    if ((long)grid * b > kLossPartials) grid = kLossPartials / b;
    if (grid < 1) return DQ_ERR_UNSUPPORTED;
    {
        LaunchScope sc(&c->prof, c->stream, DQ_K_WHIP, 8.0 * b * T * (double)n, (double)b * T * n * (4.0 + esz));
        DQ_HIP(launch_objective(objective, quant_bits, Y, ldy, T, n, scale, dY, dydt == DQ_BF16, lddy, lpart, grid,
                                c->stream, b, (long)T * ldy, (long)T * lddy));
    }
    DQ_HIP(launch_loss_finish(lpart, grid, scale, loss_dev, flags, c->stream, b));
    return DQ_OK;
}

dq_status dq_set_objective(dq_ctx* c, dq_objective objective, int quant_bits) {
    if (c == nullptr) return DQ_ERR_NULL;
    if (objective != DQ_OBJ_WHIP && objective != DQ_OBJ_VARIANCE && objective != DQ_OBJ_KURTOSIS &&
        objective != DQ_OBJ_QUANT)
        return DQ_ERR_DTYPE;
    if (quant_bits < 1 || quant_bits > 16) return DQ_ERR_SHAPE;
    c->objective = objective;
    c->quant_bits = quant_bits;
    return DQ_OK;
}

dq_status dq_set_option(dq_ctx* c, dq_option option, int value) {
    if (c == nullptr) return DQ_ERR_NULL;
    switch (option) {
        case DQ_OPT_ACCUM_PANELS:
            if (value < 0 || value > kAccumPanels) return DQ_ERR_SHAPE;
            c->accum_panels = value;
            return DQ_OK;
        case DQ_OPT_TALL_PANEL_MIN_ROWS:
            if (value < 0) return DQ_ERR_SHAPE;
            c->chol_min_m = value;
            return DQ_OK;
        case DQ_OPT_SINGLE_STREAM: c->single_stream = value != 0; return DQ_OK;
        case DQ_OPT_FUSED_WHIP: c->fused_whip = value != 0; return DQ_OK;
        case DQ_OPT_DEVICE_SYNC: c->device_sync = value != 0; return DQ_OK;
        case DQ_OPT_TWO_LEVEL_ROWS:
            if (value < -1) return DQ_ERR_SHAPE;
            c->two_level_rows = value;
            return DQ_OK;
        case DQ_OPT_FUSED_PANEL:
            if (value < 0 || value > 2) return DQ_ERR_SHAPE;
            c->fused_panel = value;
            return DQ_OK;
        case DQ_OPT_SPLIT_GEMM:
            if (value < 0 || value > 2) return DQ_ERR_SHAPE;
            c->split_gemm = value;
            return DQ_OK;
        case DQ_OPT_HEADS_BATCHED: c->heads_batched = value != 0; return DQ_OK;
    }
    return DQ_ERR_DTYPE;
}

dq_status dq_stream_handover_probe(dq_ctx* c, void* consumer_stream, void* producer_stream, int* usable) {
    if (c == nullptr || usable == nullptr) return DQ_ERR_NULL;
    if (c->ws == nullptr) return DQ_ERR_WORKSPACE;
    bool ok = false;
    DQ_HIP(handover_probe(c, static_cast<hipStream_t>(consumer_stream), static_cast<hipStream_t>(producer_stream), &ok));
    *usable = ok ? 1 : 0;
    return DQ_OK;
}

dq_status dq_qr_backward(dq_ctx* c, int b, int n, const float* R, long ldr, const float* U, long ldu, const float* G,
                         long ldg, float* dZ, long lddz) {
    if (c == nullptr) return DQ_ERR_NULL;
    if (b < 0) return DQ_ERR_SHAPE;
    DQ_TRY(check_n(n));
    DQ_TRY(check_f32(R, ldr, n));
    DQ_TRY(check_f32(U, ldu, n));
    DQ_TRY(check_f32(G, ldg, n));
    DQ_TRY(check_f32(dZ, lddz, n));
    const Layout L = make_layout(n, 1);
    DQ_TRY(check_ws(c, L));
    if (heads_route(c, n)) {
        const HeadsLayout H = make_heads_layout(L.total, b, 1);
        DQ_TRY(check_heads_ws(c, H));
        return heads_backward(c, H, b, R, ldr, U, ldu, G, ldg, dZ, lddz, nullptr, 0, 0.f);
    }
    for (int i = 0; i < b; ++i)
        DQ_TRY(qr_backward_one(c, L, n, R + (long)i * n * ldr, ldr, U + (long)i * n * ldu, ldu, G + (long)i * n * ldg,
                               ldg, dZ + (long)i * n * lddz, lddz, nullptr, 0, 0.f));
    return DQ_OK;
}

dq_status dq_hadamard_init(dq_ctx* c, int b, int n, const float* signs_dev, float* Z, long ldz) {
    if (c == nullptr || signs_dev == nullptr) return DQ_ERR_NULL;
    if (b < 0) return DQ_ERR_SHAPE;
    DQ_TRY(check_n(n));
    if ((n & (n - 1)) != 0) return DQ_ERR_UNSUPPORTED;
    DQ_TRY(check_f32(Z, ldz, n));
    for (int i = 0; i < b; ++i) {
        LaunchScope sc(&c->prof, c->stream, DQ_K_SMALL, 0.0, 4.0 * n * (double)n);
        DQ_HIP(launch_hadamard_init(signs_dev + (long)i * n, n, Z + (long)i * n * ldz, ldz, c->stream));
    }
    return DQ_OK;
}

dq_status dq_outlier_count(dq_ctx* c, int b, int T, int n, const float* Y, long ldy, float tau,
                           unsigned long long* counts_dev) {
    if (c == nullptr || counts_dev == nullptr) return DQ_ERR_NULL;
    if (b < 0 || T < 1 || n < 1) return DQ_ERR_SHAPE;
    DQ_TRY(check_f32(Y, ldy, n));
    if ((reinterpret_cast<uintptr_t>(counts_dev) & 7) != 0) return DQ_ERR_ALIGN;
    if (b == 0) return DQ_OK;
    LaunchScope sc(&c->prof, c->stream, DQ_K_SMALL, 0.0, 4.0 * b * T * (double)n);
    DQ_HIP(launch_fill_u32(reinterpret_cast<unsigned*>(counts_dev), 2L * b, 0u, c->stream));
    for (int i = 0; i < b; ++i)
        DQ_HIP(launch_outlier_count(Y + (long)i * T * ldy, ldy, T, n, tau, counts_dev + i, c->stream));
    return DQ_OK;
}

dq_status dq_gather_rows(dq_ctx* c, int b, int T_all, int T_out, int n, const void* X_all, dq_dtype dtype,
                         long ldx_all, const int* idx, void* X_out, long ldx_out) {
    if (c == nullptr || idx == nullptr) return DQ_ERR_NULL;
    if (b < 0 || T_all < 1 || T_out < 0 || n < 1) return DQ_ERR_SHAPE;
    DQ_TRY(check_x(X_all, dtype, ldx_all, n));
    DQ_TRY(check_x(X_out, dtype, ldx_out, n));
    const size_t esz = (dtype == DQ_BF16) ? 2 : 4;
    if (((size_t)n * esz) % 16 != 0) return DQ_ERR_ALIGN;
    if ((reinterpret_cast<uintptr_t>(idx) & 3) != 0) return DQ_ERR_ALIGN;
    if (c->ws == nullptr) return DQ_ERR_WORKSPACE;
    for (int i = 0; i < b; ++i) {
        LaunchScope sc(&c->prof, c->stream, DQ_K_SMALL, 0.0, 2.0 * T_out * (double)n * esz);
        DQ_HIP(launch_gather_rows(static_cast<const char*>(X_all) + (size_t)i * T_all * ldx_all * esz,
                                  (long)(ldx_all * esz), T_all, idx + (long)i * T_out, T_out, (int)(n * esz),
                                  static_cast<char*>(X_out) + (size_t)i * T_out * ldx_out * esz, (long)(ldx_out * esz),
                                  at<unsigned>(c, 0), c->stream));
    }
    return DQ_OK;
}

dq_status dq_sgd_update(dq_ctx* c, int b, int n, float* Z, long ldz, const float* dZ, long lddz, float lr) {
    if (c == nullptr) return DQ_ERR_NULL;
    if (b < 0 || n < 1) return DQ_ERR_SHAPE;
    DQ_TRY(check_f32(Z, ldz, n));
    DQ_TRY(check_f32(dZ, lddz, n));
    for (int i = 0; i < b; ++i) {
        LaunchScope sc(&c->prof, c->stream, DQ_K_SMALL, 2.0 * n * (double)n, 12.0 * n * (double)n);
        DQ_HIP(launch_axpy2d(Z + (long)i * n * ldz, ldz, dZ + (long)i * n * lddz, lddz, n, -lr, c->stream));
    }
    return DQ_OK;
}

dq_status dq_adam_update(dq_ctx* c, int b, int n, float* Z, long ldz, const float* dZ, long lddz, float* m, long ldm,
                         float* v, long ldv, int step, float lr, float beta1, float beta2, float eps) {
    if (c == nullptr) return DQ_ERR_NULL;
    if (b < 0 || n < 1 || step < 1) return DQ_ERR_SHAPE;
    DQ_TRY(check_f32(Z, ldz, n));
    DQ_TRY(check_f32(dZ, lddz, n));
    DQ_TRY(check_f32(m, ldm, n));
    DQ_TRY(check_f32(v, ldv, n));
    const float c1 = (float)(1.0 / (1.0 - pow((double)beta1, (double)step)));
    const float c2 = (float)(1.0 / (1.0 - pow((double)beta2, (double)step)));
    for (int i = 0; i < b; ++i) {
        LaunchScope sc(&c->prof, c->stream, DQ_K_SMALL, 12.0 * n * (double)n, 28.0 * n * (double)n);
        DQ_HIP(launch_adam2d(Z + (long)i * n * ldz, ldz, dZ + (long)i * n * lddz, lddz, m + (long)i * n * ldm, ldm,
                             v + (long)i * n * ldv, ldv, n, lr, beta1, beta2, eps, c1, c2, c->stream));
    }
    return DQ_OK;
}

dq_status dq_sgd_momentum_update(dq_ctx* c, int b, int n, float* Z, long ldz, const float* dZ, long lddz, float* buf,
                                 long ldbuf, float lr, float mu) {
    if (c == nullptr) return DQ_ERR_NULL;
    if (b < 0 || n < 1) return DQ_ERR_SHAPE;
    DQ_TRY(check_f32(Z, ldz, n));
    DQ_TRY(check_f32(dZ, lddz, n));
    DQ_TRY(check_f32(buf, ldbuf, n));
    for (int i = 0; i < b; ++i) {
        LaunchScope sc(&c->prof, c->stream, DQ_K_SMALL, 4.0 * n * (double)n, 20.0 * n * (double)n);
        DQ_HIP(launch_momentum2d(Z + (long)i * n * ldz, ldz, dZ + (long)i * n * lddz, lddz, buf + (long)i * n * ldbuf,
                                 ldbuf, n, lr, mu, c->stream));
    }
    return DQ_OK;
}

dq_status dq_calib_step_adam(dq_ctx* c, int b, int T, int n, const void* X, dq_dtype xdt, long ldx, float* Z, long ldz,
                             float* m, long ldm, float* v, long ldv, int step, float lr, float beta1, float beta2,
                             float eps, dq_reduce red, float* loss_dev, float* R, long ldr) {
    if (c == nullptr || loss_dev == nullptr) return DQ_ERR_NULL;
    if (b < 0 || T < 1 || step < 1) return DQ_ERR_SHAPE;
    DQ_TRY(check_n(n));
    if (red != DQ_REDUCE_TOKEN_MEAN && red != DQ_REDUCE_SUM) return DQ_ERR_DTYPE;
    DQ_TRY(check_x(X, xdt, ldx, n));
    DQ_TRY(check_f32(Z, ldz, n));
    DQ_TRY(check_f32(m, ldm, n));
    DQ_TRY(check_f32(v, ldv, n));
    if (R != nullptr) DQ_TRY(check_f32(R, ldr, n));
    const Layout L = make_layout(n, T);
    DQ_TRY(check_ws(c, L));
    const size_t esz = (xdt == DQ_BF16) ? 2 : 4;
    const float c1 = (float)(1.0 / (1.0 - pow((double)beta1, (double)step)));
    const float c2 = (float)(1.0 / (1.0 - pow((double)beta2, (double)step)));
    if (heads_fused_route(c, n) && xdt == DQ_BF16 && ldz == n && ldm == n && ldv == n) {
        const HeadsLayout H = make_heads_layout(L.total, b, T);
        DQ_TRY(check_heads_ws(c, H));
        float* Rh = R ? R : at<float>(c, H.R);
        const long ldrh = R ? ldr : kHeadDim;
        float* Uh = at<float>(c, H.U);
        float* Gh = at<float>(c, H.G);
        float* dZh = at<float>(c, H.B);   // B = R^T G is consumed before the last product writes dZ there
        DQ_TRY(heads_qr(c, b, Z, ldz, Rh, ldrh, Uh, kHeadDim));
        const bool early = !c->single_stream && b >= 1;
        if (early) DQ_TRY(heads_uinv_early(c, H, b, Uh, kHeadDim));
        DQ_TRY(heads_rotate_loss_grad(c, H, b, T, X, ldx, Rh, ldrh, red, loss_dev, Gh, kHeadDim));
        if (early) DQ_HIP(hipStreamWaitEvent(c->stream, c->sync_ev[1], 0));
        DQ_TRY(heads_backward(c, H, b, Rh, ldrh, Uh, kHeadDim, Gh, kHeadDim, dZh, kHeadDim, nullptr, 0, 0.f, early));
        // the b problems are stacked row-wise with a common row stride: one elementwise pass over b*n rows
        LaunchScope sc(&c->prof, c->stream, DQ_K_SMALL, 12.0 * b * n * (double)n, 28.0 * b * n * (double)n);
        DQ_HIP(launch_adam2d(Z, ldz, dZh, kHeadDim, m, ldm, v, ldv, n, lr, beta1, beta2, eps, c1, c2, c->stream, b * n));
        return DQ_OK;
    }
    for (int i = 0; i < b; ++i) {
        float* Zi = Z + (long)i * n * ldz;
        float* Ri = R ? R + (long)i * n * ldr : at<float>(c, L.R);
        const long ldri = R ? ldr : L.ld;
        float* Ui = at<float>(c, L.U);   // sign-normalised always, as in dq_calib_step
        float* Gi = at<float>(c, L.G);
        float* dZi = at<float>(c, L.B);   // B = R^T G is consumed before the last product writes dZ there
        const void* Xi = static_cast<const char*>(X) + (size_t)i * T * ldx * esz;
        DQ_TRY(qr_orth_one(c, L, n, Zi, ldz, Ri, ldri, Ui, L.ld));
        DQ_TRY(rotate_loss_grad_one(c, L, T, n, Xi, xdt, ldx, Ri, ldri, red, loss_dev + i, Gi, L.ld,
                                    at<float>(c, L.Y), L.ld, at<char>(c, L.dY), L.ld, false));
        DQ_TRY(qr_backward_one(c, L, n, Ri, ldri, Ui, L.ld, Gi, L.ld, dZi, L.ld, nullptr, 0, 0.f));
        LaunchScope sc(&c->prof, c->stream, DQ_K_SMALL, 12.0 * n * (double)n, 28.0 * n * (double)n);
        DQ_HIP(launch_adam2d(Zi, ldz, dZi, L.ld, m + (long)i * n * ldm, ldm, v + (long)i * n * ldv, ldv, n, lr, beta1,
                             beta2, eps, c1, c2, c->stream));
    }
    return DQ_OK;
}

dq_status dq_cayley_update(dq_ctx* c, int b, int n, float* R, long ldr, const float* G, long ldg, float* M, long ldm,
                           float lr, float beta, float q, int iters, float eps, float* alpha_dev_or_null) {
    if (c == nullptr) return DQ_ERR_NULL;
    if (b < 0 || iters < 0 || iters > 64 || !(q > 0.f) || !(eps >= 0.f)) return DQ_ERR_SHAPE;
    DQ_TRY(check_n(n));
    DQ_TRY(check_f32(R, ldr, n));
    DQ_TRY(check_f32(G, ldg, n));
    DQ_TRY(check_f32(M, ldm, n));
    const Layout L = make_layout(n, 1);
    DQ_TRY(check_ws(c, L));
    for (int i = 0; i < b; ++i)
        DQ_TRY(cayley_update_one(c, L, n, R + (long)i * n * ldr, ldr, G + (long)i * n * ldg, ldg, M + (long)i * n * ldm,
                                 ldm, lr, beta, q, iters, eps, alpha_dev_or_null ? alpha_dev_or_null + i : nullptr));
    return DQ_OK;
}

dq_status dq_cayley_step(dq_ctx* c, int b, int T, int n, const void* X, dq_dtype xdt, long ldx, float* R, long ldr,
                         float* M, long ldm, float lr, float beta, float q, int iters, float eps, dq_reduce red,
                         float* loss_dev) {
    if (c == nullptr || loss_dev == nullptr) return DQ_ERR_NULL;
    if (b < 0 || T < 1 || iters < 0 || iters > 64 || !(q > 0.f) || !(eps >= 0.f)) return DQ_ERR_SHAPE;
    DQ_TRY(check_n(n));
    if (red != DQ_REDUCE_TOKEN_MEAN && red != DQ_REDUCE_SUM) return DQ_ERR_DTYPE;
    DQ_TRY(check_x(X, xdt, ldx, n));
    DQ_TRY(check_f32(R, ldr, n));
    DQ_TRY(check_f32(M, ldm, n));
    const Layout L = make_layout(n, T);
    DQ_TRY(check_ws(c, L));
    const size_t esz = (xdt == DQ_BF16) ? 2 : 4;
    for (int i = 0; i < b; ++i) {
        float* Ri = R + (long)i * n * ldr;
        float* Gi = at<float>(c, L.G);
        const void* Xi = static_cast<const char*>(X) + (size_t)i * T * ldx * esz;
        DQ_TRY(rotate_loss_grad_one(c, L, T, n, Xi, xdt, ldx, Ri, ldr, red, loss_dev + i, Gi, L.ld, at<float>(c, L.Y),
                                    L.ld, at<char>(c, L.dY), L.ld, false));
        DQ_TRY(cayley_update_one(c, L, n, Ri, ldr, Gi, L.ld, M + (long)i * n * ldm, ldm, lr, beta, q, iters, eps, nullptr));
    }
    return DQ_OK;
}

dq_status dq_gemm_f32(dq_ctx* c, int M, int N, int K, float alpha, const float* A, long lda, int ta, const float* B,
                      long ldb, int tb, float beta, float* C, long ldc) {
    if (c == nullptr) return DQ_ERR_NULL;
    if (M < 0 || N < 0 || K < 0) return DQ_ERR_SHAPE;
    if (M == 0 || N == 0) return DQ_OK;
    DQ_TRY(check_f32(A, lda, ta ? M : K));
    DQ_TRY(check_f32(B, ldb, tb ? K : N));
    DQ_TRY(check_f32(C, ldc, N));
    GemmF32 g;
    g.A = A; g.lda = lda; g.ta = ta ? 1 : 0;
    g.B = B; g.ldb = ldb; g.tb = tb ? 1 : 0;
    g.C = C; g.ldc = ldc; g.M = M; g.N = N; g.K = K; g.alpha = alpha; g.beta = beta;
    LaunchScope sc(&c->prof, c->stream, DQ_K_GEMM_F32, 2.0 * M * (double)N * K, 0.0);
    DQ_HIP(launch_gemm_f32(g, c->stream));
    return DQ_OK;
}

dq_status dq_gemm_bf16(dq_ctx* c, int M, int N, int K, const void* A, long lda, int ta, const void* B, long ldb,
                       int tb, float* C, long ldc) {
    if (c == nullptr) return DQ_ERR_NULL;
    if (M < 0 || N < 0 || K < 0) return DQ_ERR_SHAPE;
    if (M == 0 || N == 0) return DQ_OK;
    DQ_TRY(check_bf16(A, lda, ta ? M : K));
    DQ_TRY(check_bf16(B, ldb, tb ? K : N));
    DQ_TRY(check_f32(C, ldc, N));
    GemmBf16 g;
    g.A = static_cast<const bf16_t*>(A); g.lda = lda; g.ta = ta ? 1 : 0;
    g.B = static_cast<const bf16_t*>(B); g.ldb = ldb; g.tb = tb ? 1 : 0;
    g.C = C; g.ldc = ldc; g.M = M; g.N = N; g.K = K;
    LaunchScope sc(&c->prof, c->stream, DQ_K_GEMM_BF16, 2.0 * M * (double)N * K, 0.0);
    DQ_HIP(launch_gemm_bf16(g, c->stream));
    return DQ_OK;
}

dq_status dq_profile_enable(dq_ctx* c, unsigned mask) {
    if (c == nullptr) return DQ_ERR_NULL;
    DQ_HIP(hipStreamSynchronize(c->stream));
    c->prof.mask = mask;
    c->prof.recs.clear();
    c->prof.failed = false;
    return DQ_OK;
}

dq_status dq_profile_read(dq_ctx* c, dq_kernel_class k, double* ms, long* launches, double* flops, double* bytes) {
    if (c == nullptr) return DQ_ERR_NULL;
    if ((int)k < 0 || (int)k >= DQ_K_COUNT) return DQ_ERR_DTYPE;
    DQ_HIP(hipStreamSynchronize(c->stream));
    if (c->prof.failed) return DQ_ERR_HIP;
    double tms = 0.0, tf = 0.0, tb = 0.0;
    long cnt = 0;
    for (size_t i = 0; i < c->prof.recs.size(); ++i) {
        if (c->prof.recs[i].klass != (int)k) continue;
        float one = 0.f;
        DQ_HIP(hipEventElapsedTime(&one, c->prof.ev[2 * i], c->prof.ev[2 * i + 1]));
        tms += one; tf += c->prof.recs[i].flops; tb += c->prof.recs[i].bytes; ++cnt;
    }
    if (ms) *ms = tms;
    if (launches) *launches = cnt;
    if (flops) *flops = tf;
    if (bytes) *bytes = tb;
    return DQ_OK;
}

}  // extern "C"
