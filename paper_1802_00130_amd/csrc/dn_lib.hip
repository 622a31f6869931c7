// libdn: host side of the C-ABI declared in include/dn.h.  Validates arguments, lays out the
// caller's workspace, and enqueues the HIP kernels of dn_gemm.h / dn_kernels.h on one stream.
#include "../../include/dn.h"

#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstdint>
#include <cstdlib>
#include <cstring>
#include <new>
#include <vector>

#include "dn_gemm.h"
#include "dn_kernels.h"

using namespace dn;

namespace {

constexpr int kTargetWGs = 1024;  // ~4 work-groups per compute unit (256 CUs)
// K-tile depths; slices of split sums are cut at multiples of the deepest
constexpr int kBKmax = 32;
// tile rows per super-row of the tile walk: 8 x 8 tiles are about what one XCD (32 CUs) holds at a time
constexpr int kGroupM = 8;
// most work-groups of 256 threads a launch can have resident on the chip (256 CUs x 2048 threads / 256);
// sizes the exchange buffers of the team kernel
constexpr int kMaxResidentWGs = 2048;
// 64-bit words in each exchange region of the team kernel: teams x 2 sets x (work-groups per team) x
// (at most 128 rows per work-group), teams x work-groups <= kMaxResidentWGs
constexpr long long kTeamExchWords = 2LL * kMaxResidentWGs * 128;

enum KernelClass {
    KC_GEMM_FWD = 0,      // forward layer products (all samples or subsample)
    KC_GEMM_BACK,         // back-propagation of delta
    KC_GEMM_TN_GRAD,      // gradient sums over samples
    KC_GEMM_PREP,         // Jacobian backward sweeps
    KC_GEMM_Q,            // product: inner sums over t (Z V)
    KC_GEMM_TN_MATVEC,    // product: sums over samples (T^T Z)
    KC_JV_JTV_FUSED,      // product: both passes over P, one read
    KC_JV,                // product: P q
    KC_JTV,               // product: P^T r
    KC_JV_JTV_TEAM,       // product: both passes over P, one read, teams of work-groups
    KC_GEMM_IMPLICIT,     // product: the two small dense products that stand in for block L-1
    KC_GEMM_ROP,          // product without stored blocks: forward-mode and back-propagation sweeps
    KC_TN_REDUCE,         // slice fold + regularisation term
    KC_JAC_INIT,
    KC_GATHER,
    KC_LOSS,
    KC_CG_VEC,
    KC_COUNT
};

const char* const kClassNames[KC_COUNT] = {
    "gemm_forward", "gemm_backprop", "gemm_tn_grad", "gemm_jacobian_prep", "gemm_q_matvec", "gemm_tn_matvec",
    "jv_jtv_fused", "jv_rows", "jtv_cols", "jv_jtv_team", "gemm_implicit_block", "gemm_rop_sweeps", "tn_reduce", "jac_init", "gather_rows", "loss", "cg_vector"};

inline long long round_up(long long x, long long a) { return (x + a - 1) / a * a; }
inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
inline int cdiv(long long a, long long b) { return (int)((a + b - 1) / b); }

struct TnPlan {
    int tile;                       // 64 or 128
    int splits;
    int k_per_split;
    long long floats[DN_MAX_LAYERS + 1];  // per layer, floats of partial storage
    long long offset[DN_MAX_LAYERS + 1];  // per layer, offset in the partial buffer
    long long total;
};

}  // namespace

struct dn_ctx {
    int L = 0;
    int dims[DN_MAX_LAYERS + 1] = {0};
    double C = 1.0;
    int l_max = 0, s_max = 0;
    long long n = 0;
    long long woff[DN_MAX_LAYERS + 1] = {0}, boff[DN_MAX_LAYERS + 1] = {0};
    long long ld[DN_MAX_LAYERS + 1] = {0};    // padded row stride of layer-m activations
    long long ldw[DN_MAX_LAYERS + 1] = {0};   // padded row stride of the sum-over-samples partials
    long long ldr = 0;

    // workspace layout (byte offsets)
    size_t ws_bytes = 0;
    size_t o_Zall[DN_MAX_LAYERS + 1] = {0};
    size_t o_D[2] = {0, 0};
    size_t o_ZS[DN_MAX_LAYERS + 1] = {0};
    size_t o_P[DN_MAX_LAYERS + 1] = {0};
    size_t o_Q[DN_MAX_LAYERS + 1] = {0};
    size_t o_Qb = 0;           // second half of one layer's Q when its sum over t is cut in two
    size_t o_T[DN_MAX_LAYERS + 1] = {0};
    size_t o_AL = 0;
    size_t o_thS = 0;          // copy of theta taken by dn_jacobian_prep (the product without stored blocks needs A^m)
    size_t o_WT = 0;           // W^m = (A^m)^T for m = 2..L, dense, at the theta offsets of A^m
    size_t o_R = 0, o_tn = 0, o_r = 0, o_p = 0, o_q = 0, o_part[3] = {0, 0, 0}, o_state = 0, o_f = 0;
    // outer Newton iteration: gradient, direction, G d, G d_prev, trial point; partial sums of 5 dot products
    size_t o_ng = 0, o_nd = 0, o_nGd = 0, o_nGdb = 0, o_ntheta = 0, o_npart = 0;
    // team kernel: partial vectors, folded vectors, counters, error word
    size_t o_texch = 0, o_terr = 0, o_ttp[DN_MAX_LAYERS + 1] = {0};
    // split structure (DN_PARTITION): per input group Q^{m,a} / T^{m,a}, per partition r, the index map that
    // lists theta partition by partition, CG vectors in that order and theta-layout operands of the product
    size_t o_Qp[DN_MAX_LAYERS + 1] = {0}, o_Tp[DN_MAX_LAYERS + 1] = {0}, o_Rp = 0, o_perm = 0, o_gperm = 0,
           o_dperm = 0, o_ptheta = 0, o_qtheta = 0;
    int split[DN_MAX_LAYERS + 1] = {0};
    int gbound[DN_MAX_LAYERS + 1][DN_MAX_SPLIT + 1] = {{0}};   // first neuron of each group
    int part_base[DN_MAX_LAYERS + 2] = {0};
    int nparts = 0;
    long long part_off[DN_MAX_SEGS + 1] = {0};   // partition k covers [part_off[k], part_off[k+1]) of the index map
    bool split_set = false;
    int team_rpt = 0;               // rows per thread of the team kernel for this n_L (0: team kernel not applicable)
    int team_nrs = 0;               // row slices
    long long tn_floats = 0;

    char* ws = nullptr;
    hipStream_t stream = nullptr;
    bool bound = false;
    bool prepped = false;
    int s_cur = 0;
    int last_hip = 0;
    int num_cus = 256;
    // team kernel (single pass over the stored blocks for n_L > 16)
    int stream_passes = 0;          // 0 automatic, 2 force the two-pass kernels
    unsigned spin_limit = 1u << 20;
    bool team_clean = false;        // exchange words and error word cleared since the last dn_bind
    bool team_used = false;
    unsigned team_seq = 0;          // sequence numbers handed out so far
    int team_wgs_per_cu = 0;        // resident work-groups per CU of the kernel variant (0: not looked up)

    // profiling
    bool prof = false;
    unsigned long long prof_mask = ~0ull;
    double prof_ms[KC_COUNT] = {0};
    long long prof_n[KC_COUNT] = {0};
    struct Pending { int cls; hipEvent_t a, b; };
    std::vector<Pending> pending;
    std::vector<hipEvent_t> free_events;

    float* fptr(size_t off) const { return reinterpret_cast<float*>(ws + off); }
    double* dptr(size_t off) const { return reinterpret_cast<double*>(ws + off); }
};

namespace {

#define DN_HIP(ctx, expr)                                  \
    do {                                                   \
        hipError_t e__ = (expr);                           \
        if (e__ != hipSuccess) {                           \
            (ctx)->last_hip = (int)e__;                    \
            return DN_EHIP;                                \
        }                                                  \
    } while (0)

// ---- profiling ---------------------------------------------------------------------------

hipError_t prof_fold(dn_ctx* c) {
    if (c->pending.empty()) return hipSuccess;
    hipError_t e = hipStreamSynchronize(c->stream);
    if (e != hipSuccess) return e;
    for (auto& p : c->pending) {
        float ms = 0.f;
        e = hipEventElapsedTime(&ms, p.a, p.b);
        if (e != hipSuccess) return e;
        c->prof_ms[p.cls] += ms;
        c->prof_n[p.cls] += 1;
        c->free_events.push_back(p.a);
        c->free_events.push_back(p.b);
    }
    c->pending.clear();
    return hipSuccess;
}

hipError_t prof_event(dn_ctx* c, hipEvent_t* ev) {
    if (!c->free_events.empty()) {
        *ev = c->free_events.back();
        c->free_events.pop_back();
        return hipSuccess;
    }
    // no system-scope fence at the record: the bracket should perturb the stream as little as possible
    return hipEventCreateWithFlags(ev, hipEventDisableSystemFence);
}

struct ProfScope {
    dn_ctx* c;
    int cls;
    hipEvent_t a = nullptr, b = nullptr;
    hipError_t err = hipSuccess;
    bool on = false;
    ProfScope(dn_ctx* ctx, int k) : c(ctx), cls(k) {
        on = c->prof && ((c->prof_mask >> k) & 1ull);
        if (!on) return;
        if (c->pending.size() >= 4096) err = prof_fold(c);
        if (err == hipSuccess) err = prof_event(c, &a);
        if (err == hipSuccess) err = prof_event(c, &b);
        if (err == hipSuccess) err = hipEventRecord(a, c->stream);
    }
    hipError_t end() {
        if (!on || err != hipSuccess) return err;
        err = hipEventRecord(b, c->stream);
        if (err == hipSuccess) c->pending.push_back({cls, a, b});
        return err;
    }
};

// ---- GEMM plumbing -----------------------------------------------------------------------

GemmProblem mk_problem(const float* A, long long lda, const float* B, long long ldb, float* Cc, long long ldc, int M,
                       int N, int K) {
    GemmProblem p;
    std::memset(&p, 0, sizeof(p));
    p.A = A; p.B = B; p.C = Cc;
    p.lda = lda; p.ldb = ldb; p.ldc = ldc;
    p.M = M; p.N = N; p.K = K;
    p.auxdiv = 1;
    p.alpha = 1.0f;
    p.splits = 1;
    p.k_per_split = K;
    return p;
}

// Fill tile counts and the tile walk.  splits applies to every problem of the group.
void finalize_group(GemmGroup& g, int BM, int BN, int BK, int splits) {
    int begin = 0;
    for (int i = 0; i < g.nprob; ++i) {
        GemmProblem& p = g.p[i];
        p.tiles_m = cdiv(p.M, BM);
        p.tiles_n = cdiv(p.N, BN);
        p.splits = splits;
        p.k_per_split = (int)round_up(cdiv(p.K, splits), BK);
        p.tile_begin = begin;
        begin += p.tiles_m * p.tiles_n;
    }
    g.tiles_per_split = begin;
    g.total_tiles = begin * splits;
    g.group_m = kGroupM;
    g.grid = g.total_tiles;
    if (splits > 1 || g.nprob == 1) {
        g.xcd_mode = XCD_RANGES;
    } else {
        g.xcd_mode = XCD_PER_PROBLEM;
        int most = 0;
        for (int x = 0; x < kXcds; ++x) {
            int mine = 0;
            for (int i = 0; i < g.nprob; ++i) {
                const int tiles = g.p[i].tiles_m * g.p[i].tiles_n;
                mine += tiles / kXcds + (x < tiles % kXcds ? 1 : 0);
            }
            most = std::max(most, mine);
        }
        g.grid = kXcds * most;
    }
}

int group_tiles(const GemmGroup& g, int BM, int BN) {
    int t = 0;
    for (int i = 0; i < g.nprob; ++i) t += cdiv(g.p[i].M, BM) * cdiv(g.p[i].N, BN);
    return t;
}

template <int BM, int BN, int BK, int PF, int LA, int LB, int CLS, bool PIN = false>
hipError_t launch_gemm_t(const GemmGroup& g, hipStream_t st) {
    if (g.total_tiles <= 0) return hipSuccess;
    hipLaunchKernelGGL((gemm_kernel<BM, BN, BK, 2, 2, LA, LB, PF, PIN, CLS>), dim3(g.grid), dim3(256), 0, st, g);
    return hipGetLastError();
}

// Tile variants (measured on MI355X):
//   128x128, K-tile 16, 2 tiles in flight             large products of K-contiguous operands (>= 1024 tiles)
//   64x64,   K-tile 16, 4 in flight, pinned schedule  launches of <= 4 work-groups per CU, and sums over samples
//   64x64,   K-tile 16, 4 in flight                   everything else
template <int LA, int LB, int CLS>
hipError_t launch_gemm(GemmGroup& g, int tile, int splits, hipStream_t st) {
    if (tile == 128) {
        finalize_group(g, 128, 128, 16, splits);
        return launch_gemm_t<128, 128, 16, 2, LA, LB, CLS>(g, st);
    }
    finalize_group(g, 64, 64, 16, splits);
    // the hand-placed schedule wins for small launches, and at every size when both operands go through
    // the transposing loads (sums over samples)
    if (g.total_tiles <= 4 * 256 || (LA == RT && LB == RT)) return launch_gemm_t<64, 64, 16, 4, LA, LB, CLS, true>(g, st);
    return launch_gemm_t<64, 64, 16, 4, LA, LB, CLS>(g, st);
}

// Measured on MI355X: 64x64 tiles win on every shape of the path except products with both operands
// K-contiguous and both output dimensions >= 1024, where 128x128 tiles are ~5% faster once there are
// >= 4 of them per CU.
int pick_tile(const GemmGroup& g, bool both_k_contiguous) {
    if (!both_k_contiguous || group_tiles(g, 128, 128) < 1024) return 64;
    for (int i = 0; i < g.nprob; ++i)
        if (g.p[i].M < 1024 || g.p[i].N < 1024) return 64;
    return 128;
}

// K-slices of a sum over samples: enough to give every CU about 4 work-groups, at least 256 samples per
// slice.  From 6 slices on the count is rounded to a multiple of 8: the tile walk hands each XCD a
// contiguous eighth of the launch, and with 8 k slices that is exactly k whole slices, read once into that
// XCD's L2 (measured at 784-300-300-10, |S| = 3000: 10 slices 37.3 us, 8 slices 33.0 us, 16 slices 36.9 us).
int pick_splits(int tiles, int K) {
    int s = std::max(1, kTargetWGs / std::max(1, tiles));
    s = std::min(s, std::max(1, K / 256));
    s = std::min(s, 64);
    if (s >= 6) s = std::max(8, (s + 4) / 8 * 8);
    return s;
}

// Plan of the sums over samples  W_m = T^m^T [Z^{m-1}, 1]  for K samples.  grouped: all layers in
// one launch (product); otherwise one launch per layer (gradient).
TnPlan plan_tn(const dn_ctx* c, int K, bool grouped, int only_layer) {
    TnPlan pl;
    std::memset(&pl, 0, sizeof(pl));
    int tiles = 0;
    for (int m = 1; m <= c->L; ++m) {
        if (!grouped && m != only_layer) continue;
        tiles += cdiv(c->dims[m], 64) * cdiv(c->dims[m - 1] + 1, 64);
    }
    pl.tile = 64;
    pl.splits = pick_splits(tiles, K);
    pl.k_per_split = (int)round_up(cdiv(K, pl.splits), kBKmax);
    long long off = 0;
    for (int m = 1; m <= c->L; ++m) {
        pl.offset[m] = off;
        pl.floats[m] = (long long)pl.splits * c->dims[m] * c->ldw[m];
        off += round_up(pl.floats[m], 64);
    }
    pl.total = off;
    return pl;
}

size_t take(size_t& cur, size_t bytes) {
    size_t o = cur;
    cur += (size_t)round_up((long long)bytes, 256);
    return o;
}

void layout_workspace(dn_ctx* c) {
    size_t cur = 0;
    const int L = c->L;
    for (int m = 1; m <= L; ++m) c->o_Zall[m] = take(cur, sizeof(float) * (size_t)c->l_max * c->ld[m]);
    long long ldmax = 0;
    for (int m = 1; m <= L; ++m) ldmax = std::max(ldmax, c->ld[m]);
    for (int k = 0; k < 2; ++k) c->o_D[k] = take(cur, sizeof(float) * (size_t)c->l_max * ldmax);
    for (int m = 0; m <= L; ++m) c->o_ZS[m] = take(cur, sizeof(float) * (size_t)c->s_max * c->ld[m]);
    for (int m = 1; m < L; ++m) c->o_P[m] = take(cur, sizeof(float) * (size_t)c->s_max * c->dims[L] * c->ld[m]);
    for (int m = 1; m <= L; ++m) c->o_Q[m] = take(cur, sizeof(float) * (size_t)c->s_max * c->ld[m]);
    for (int m = 1; m <= L; ++m) c->o_T[m] = take(cur, sizeof(float) * (size_t)c->s_max * c->ld[m]);
    {
        long long ldmax = 0;
        for (int m = 1; m <= L; ++m) ldmax = std::max(ldmax, c->ld[m]);
        c->o_Qb = take(cur, sizeof(float) * (size_t)c->s_max * ldmax);
    }
    c->o_AL = take(cur, sizeof(float) * (size_t)c->dims[L] * c->ld[L >= 2 ? L - 1 : 0]);
    c->o_WT = take(cur, sizeof(float) * (size_t)round_up(c->n, 64));
    c->o_thS = take(cur, sizeof(float) * (size_t)round_up(c->n, 64));
    c->o_R = take(cur, sizeof(float) * (size_t)L * c->s_max * c->ldr);
    long long tn = plan_tn(c, c->s_max, true, 0).total;
    for (int m = 1; m <= L; ++m) tn = std::max(tn, plan_tn(c, c->l_max, false, m).total);
    c->tn_floats = tn;
    c->o_tn = take(cur, sizeof(float) * (size_t)tn);
    const size_t nvec = sizeof(float) * (size_t)round_up(c->n, 64);
    c->o_r = take(cur, nvec);
    c->o_p = take(cur, nvec);
    c->o_q = take(cur, nvec);
    for (int k = 0; k < 3; ++k) c->o_part[k] = take(cur, sizeof(double) * DN_MAX_PARTIALS);
    c->o_state = take(cur, 2 * sizeof(CgState));
    c->o_f = take(cur, 256);
    c->o_ng = take(cur, nvec);
    c->o_nd = take(cur, nvec);
    c->o_nGd = take(cur, nvec);
    c->o_nGdb = take(cur, nvec);
    c->o_ntheta = take(cur, nvec);
    c->o_npart = take(cur, sizeof(double) * 5 * DN_MAX_PARTIALS);
    // team kernel: exchange words (two regions of kTeamExchWords 64-bit words: partial vectors, folded
    // vectors) and, with several row slices, the per-slice partial transposed products
    c->team_rpt = 0;
    c->team_nrs = 0;
    if (L >= 3 && c->dims[L] > 16) {
        c->team_rpt = round_up(c->dims[L], 32) <= 64 ? 16 : 32;
        c->team_nrs = cdiv(c->dims[L], 4 * c->team_rpt);
        c->o_texch = take(cur, sizeof(unsigned long long) * 2 * kTeamExchWords);
        if (c->team_nrs > 1)
            for (int m = 1; m + 1 < L; ++m)
                c->o_ttp[m] = take(cur, sizeof(float) * (size_t)c->team_nrs * c->s_max * c->ld[m]);
    }
    c->o_terr = take(cur, 256);
    for (int m = 1; m <= L; ++m) {
        c->o_Qp[m] = take(cur, sizeof(float) * (size_t)DN_MAX_SPLIT * c->s_max * c->ld[m]);
        c->o_Tp[m] = take(cur, sizeof(float) * (size_t)DN_MAX_SPLIT * c->s_max * c->ld[m]);
    }
    c->o_Rp = take(cur, sizeof(float) * (size_t)DN_MAX_SPLIT * DN_MAX_SPLIT * std::max(1, L - 1) * c->s_max * c->ldr);
    c->o_perm = take(cur, sizeof(int) * (size_t)round_up(c->n, 64));
    c->o_gperm = take(cur, nvec);
    c->o_dperm = take(cur, nvec);
    c->o_ptheta = take(cur, nvec);
    c->o_qtheta = take(cur, nvec);
    c->ws_bytes = cur;
}

int grid_for(long long total, int per_block = 256 * 8);

// W^m = (A^m)^T for layers m_lo..m_hi into the workspace
int transpose_weights(dn_ctx* c, const float* theta, int m_lo, int m_hi) {
    for (int m = m_lo; m <= m_hi; ++m) {
        const int rows = c->dims[m], cols = c->dims[m - 1];
        hipLaunchKernelGGL(transpose_kernel, dim3(cdiv(cols, 32), cdiv(rows, 32)), dim3(256), 0, c->stream,
                           theta + c->woff[m], c->fptr(c->o_WT) + c->woff[m], rows, cols);
        DN_HIP(c, hipGetLastError());
    }
    return DN_OK;
}

int grid_for(long long total, int per_block) {
    long long b = (total + per_block - 1) / per_block;
    return (int)std::max<long long>(1, std::min<long long>(b, 256 * 16));
}

// ---- forward pass on `rows` rows: Zin -> Z[1..upto] ---------------------------------------
int forward_layers(dn_ctx* c, const float* theta, const float* Z0, long long ld0, int rows, const size_t* o_Z,
                   int upto) {
    const float* zin = Z0;
    long long ldin = ld0;
    for (int m = 1; m <= upto; ++m) {
        GemmGroup g;
        g.nprob = 1;
        float* zout = c->fptr(o_Z[m]);
        g.p[0] = mk_problem(zin, ldin, theta + c->woff[m], c->dims[m - 1], zout, c->ld[m], rows, c->dims[m],
                            c->dims[m - 1]);
        g.p[0].bias = theta + c->boff[m];
        const int tile = pick_tile(g, true);
        ProfScope ps(c, KC_GEMM_FWD);
        DN_HIP(c, ps.err);
        g.p[0].sigmoid = m < c->L ? 1 : 0;
        DN_HIP(c, (launch_gemm<KC, KC, KC_GEMM_FWD>(g, tile, 1, c->stream)));
        DN_HIP(c, ps.end());
        zin = zout;
        ldin = c->ld[m];
    }
    return DN_OK;
}

// objective from Z^L of all rows; optionally writes the gradient seed 2(z^L - y)
// Loss terms of the `rows` samples whose outputs are in Z^L of the workspace (one chunk of the l samples);
// optionally the gradient seed 2(z^L - y) and a dense copy of z^L.  first: this is the first chunk (the
// partial sums start from zero).  last && f_host: add the regularisation term and return f.
int objective(dn_ctx* c, const float* theta, const float* Y, int rows, int l, bool first, bool last, float* delta,
              long long ldd, float* zl_out, double* f_host) {
    const int L = c->L;
    // the grid of the first (largest) chunk defines how many partial sums there are
    const int nb_all = std::min(DN_MAX_PARTIALS, grid_for((long long)std::min(l, c->l_max) * c->dims[L]));
    const int nb_loss = std::min(nb_all, grid_for((long long)rows * c->dims[L]));
    const int nb_reg = std::min(DN_MAX_PARTIALS, grid_for(c->n));
    ProfScope ps(c, KC_LOSS);
    DN_HIP(c, ps.err);
    hipLaunchKernelGGL(loss_delta_kernel, dim3(nb_loss), dim3(256), 0, c->stream, c->fptr(c->o_Zall[L]), c->ld[L], Y,
                       rows, c->dims[L], delta, ldd, zl_out, c->dptr(c->o_part[0]), first ? 0 : 1);
    DN_HIP(c, hipGetLastError());
    if (f_host && last) {
        hipLaunchKernelGGL(sumsq_kernel, dim3(nb_reg), dim3(256), 0, c->stream, theta, c->n, c->dptr(c->o_part[1]));
        DN_HIP(c, hipGetLastError());
        hipLaunchKernelGGL(objective_finalize_kernel, dim3(1), dim3(256), 0, c->stream, c->dptr(c->o_part[0]),
                           nb_all, c->dptr(c->o_part[1]), nb_reg, 1.0 / (2.0 * c->C), 1.0 / (double)l,
                           c->dptr(c->o_f));
        DN_HIP(c, hipGetLastError());
    }
    DN_HIP(c, ps.end());
    if (f_host && last) {
        DN_HIP(c, hipMemcpyAsync(f_host, c->dptr(c->o_f), sizeof(double), hipMemcpyDeviceToHost, c->stream));
        DN_HIP(c, hipStreamSynchronize(c->stream));
    }
    return DN_OK;
}

// out = x/C + scale * (folded partial sums), theta layout
int tn_reduce(dn_ctx* c, const TnPlan* plans /* indexed by layer, or one plan for all */, bool per_layer,
              const float* x, float* out, double scale) {
    ReduceArgs ra;
    std::memset(&ra, 0, sizeof(ra));
    ra.L = c->L;
    for (int m = 0; m <= c->L; ++m) ra.n[m] = c->dims[m];
    int blocks = 0;
    for (int m = 1; m <= c->L; ++m) {
        const TnPlan& pl = per_layer ? plans[m] : plans[0];
        ra.off[m] = c->woff[m];
        ra.W[m] = c->fptr(c->o_tn) + pl.offset[m];
        ra.ldw[m] = c->ldw[m];
        ra.split_stride[m] = (long long)c->dims[m] * c->ldw[m];
        ra.splits[m] = pl.splits;
        ra.chunks[m] = cdiv(c->dims[m - 1] + 1, 1024);
        ra.blk_begin[m] = blocks;
        blocks += c->dims[m] * ra.chunks[m];
    }
    ra.blk_begin[c->L + 1] = blocks;
    ProfScope ps(c, KC_TN_REDUCE);
    DN_HIP(c, ps.err);
    hipLaunchKernelGGL(tn_reduce_kernel, dim3(blocks), dim3(256), 0, c->stream, ra, x, out, (float)(1.0 / c->C),
                       (float)scale);
    DN_HIP(c, hipGetLastError());
    DN_HIP(c, ps.end());
    return DN_OK;
}

void fill_stream_args(const dn_ctx* c, StreamArgs& a, int mode) {
    std::memset(&a, 0, sizeof(a));
    a.L = c->L;
    a.s = c->s_cur;
    a.nL = c->dims[c->L];
    a.blockdiag = mode == DN_BLOCKDIAG ? 1 : 0;
    for (int m = 0; m <= c->L; ++m) {
        a.n[m] = c->dims[m];
        a.ld[m] = c->ld[m];
    }
    for (int m = 1; m < c->L; ++m) a.P[m] = c->fptr(c->o_P[m]);
    for (int m = 1; m <= c->L; ++m) {
        a.Q[m] = c->fptr(c->o_Q[m]);
        a.T[m] = c->fptr(c->o_T[m]);
    }
    a.R = c->fptr(c->o_R);
    a.ldr = c->ldr;
    int w = 0;
    for (int m = 1; m < c->L; ++m)
        for (int cidx = 0; cidx < cdiv(c->dims[m], 256); ++cidx, ++w)
            if (w < DN_MAX_WSLOTS) {
                a.wlayer[w] = m;
                a.wcol[w] = cidx;
            }
    a.nwslots = w;
}

// ---- team kernel plumbing ------------------------------------------------------------------
struct TeamPlan {
    bool ok = false;
    TeamArgs ta;
};

hipError_t plan_team(dn_ctx* c, const StreamArgs& a, TeamPlan& tp) {
    tp.ok = false;
    const int L = c->L;
    if (c->stream_passes == 2 || c->team_rpt == 0) return hipSuccess;
    if (c->team_wgs_per_cu == 0) {
        int nb = 0;
        hipError_t e = c->team_rpt == 16
                           ? hipOccupancyMaxActiveBlocksPerMultiprocessor(&nb, jv_jtv_team_kernel<16, 0, 4>, 256, 0)
                           : hipOccupancyMaxActiveBlocksPerMultiprocessor(&nb, jv_jtv_team_kernel<32, 8, 3>, 256, 0);
        if (e != hipSuccess) return e;
        c->team_wgs_per_cu = nb >= 1 ? nb : -1;
    }
    if (c->team_wgs_per_cu < 1) return hipSuccess;
    TeamArgs& ta = tp.ta;
    std::memset(&ta, 0, sizeof(ta));
    ta.a = a;
    const int RB = 4 * c->team_rpt;
    int ncs = 0;
    for (int m = 1; m + 1 < L; ++m) {
        ta.slice_begin[m] = ncs;
        ncs += cdiv(c->dims[m], 256);
    }
    const int G = c->team_nrs * ncs;
    const int resident = std::min(kMaxResidentWGs, c->num_cus * c->team_wgs_per_cu);
    const int teams = std::min(a.s, resident / G);
    if (teams < 1) return hipSuccess;
    ta.G = G;
    ta.teams = teams;
    ta.nrs = c->team_nrs;
    ta.ncs = ncs;
    ta.ntasks = (RB / 32) * ta.nrs * (a.blockdiag ? (L - 2) : 1);
    ta.nfolders = std::min(G, ta.ntasks);
    ta.part = reinterpret_cast<unsigned long long*>(c->ws + c->o_texch);
    ta.rbar = ta.part + kTeamExchWords;
    for (int m = 1; m + 1 < L; ++m) ta.tpart[m] = c->team_nrs > 1 ? c->fptr(c->o_ttp[m]) : nullptr;
    ta.error = reinterpret_cast<unsigned*>(c->ws + c->o_terr);
    ta.spin_limit = c->spin_limit;
    tp.ok = true;
    return hipSuccess;
}

hipError_t launch_team(dn_ctx* c, TeamPlan& tp) {
    TeamArgs& ta = tp.ta;
    const unsigned per_launch = (unsigned)cdiv(ta.a.s, ta.teams) + 1u;
    if (!c->team_clean || c->team_seq > 0x7fff0000u) {
        // first use after dn_bind (or the sequence numbers are about to wrap): start from a blank slate
        hipLaunchKernelGGL(team_clear_kernel, dim3(1024), dim3(256), 0, c->stream, ta.part, 2 * kTeamExchWords,
                           ta.error);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
        c->team_clean = true;
        c->team_seq = 0;
    }
    ta.seq_base = c->team_seq;
    c->team_seq += per_launch;
    c->team_used = true;
    const dim3 grid(ta.teams * ta.G), block(256);
    if (c->team_rpt == 16) hipLaunchKernelGGL((jv_jtv_team_kernel<16, 0, 4>), grid, block, 0, c->stream, ta);
    else                   hipLaunchKernelGGL((jv_jtv_team_kernel<32, 8, 3>), grid, block, 0, c->stream, ta);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || ta.nrs == 1) return e;
    // several row slices: add their partial transposed products
    for (int m = 1; m + 1 < c->L; ++m) {
        const long long total4 = (long long)ta.a.s * c->ld[m] / 4;
        hipLaunchKernelGGL(team_fold_t_kernel, dim3(grid_for(total4, 256 * 4)), dim3(256), 0, c->stream, ta.tpart[m],
                           c->fptr(c->o_T[m]), ta.nrs, total4);
        e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

// after a synchronisation: has a wait of the team kernel run out?
int team_status(dn_ctx* c) {
    if (!c->team_used) return DN_OK;
    unsigned err = 0;
    DN_HIP(c, hipMemcpyAsync(&err, c->ws + c->o_terr, sizeof(err), hipMemcpyDeviceToHost, c->stream));
    DN_HIP(c, hipStreamSynchronize(c->stream));
    return err ? DN_ETIMEOUT : DN_OK;
}

int gn_matvec_part(dn_ctx* c, const float* v, float* out);

// out = G^S v (mode full / per-layer), Section 4.2 factored products on the stored blocks
int gn_matvec(dn_ctx* c, const float* v, float* out, int mode) {
    if (mode == DN_PARTITION) return c->split_set ? gn_matvec_part(c, v, out) : DN_ESTATE;
    const int L = c->L, s = c->s_cur, nL = c->dims[L];
    StreamArgs a;
    fill_stream_args(c, a, mode);
    const bool fused = L >= 2 && ((nL <= 16 && a.nwslots <= 16) || (nL <= 12 && a.nwslots <= DN_MAX_WSLOTS));
    const bool bd = mode == DN_BLOCKDIAG;
    // 1. inner sums over t for every layer: Q^m = Z^{m-1} V^m + vb^m.  On the two-pass path the
    //    last hidden layer's result is scaled by sigma'(s^{L-1}) on the way out (it is only ever used
    //    as A^L (sigma' * q^{L-1})).
    {
        GemmGroup g;
        g.nprob = L;
        for (int m = 1; m <= L; ++m) {
            g.p[m - 1] = mk_problem(c->fptr(c->o_ZS[m - 1]), c->ld[m - 1], v + c->woff[m], c->dims[m - 1],
                                    c->fptr(c->o_Q[m]), c->ld[m], s, c->dims[m], c->dims[m - 1]);
            g.p[m - 1].bias = v + c->boff[m];
            if (!fused && L >= 2 && m == L - 1) {
                g.p[m - 1].aux = c->fptr(c->o_ZS[L - 1]);
                g.p[m - 1].ldaux = c->ld[L - 1];
            }
        }
        const int tile = pick_tile(g, true);
        // Small launches (a few tiles per CU) whose longest sum over t is at least twice any other: cut that
        // layer's sum in two halves, written to Q^m and a second buffer that the fused kernel adds on the way
        // in.  The launch then consists of tiles of similar length (measured at 784-300-300-10, |S| = 3000:
        // 30.2 -> 26.8 us).
        if (fused && tile == 64 && L < DN_MAX_GROUP && group_tiles(g, 64, 64) <= 3 * c->num_cus) {
            int big = 0;                       // among the hidden layers: Q^L is read as it is
            for (int k = 1; k + 1 < L; ++k)
                if (g.p[k].K > g.p[big].K) big = k;
            int other = 0;
            for (int k = 0; k < L; ++k)
                if (k != big) other = std::max(other, g.p[k].K);
            if (g.p[big].K >= 512 && g.p[big].K >= 2 * other) {
                const int kh = (int)round_up(g.p[big].K / 2, 16);
                GemmProblem& second = g.p[g.nprob++];
                second = g.p[big];
                second.A += kh;
                second.B += kh;
                second.K -= kh;
                second.C = c->fptr(c->o_Qb);
                second.bias = nullptr;
                g.p[big].K = kh;
                a.Qb[big + 1] = c->fptr(c->o_Qb);
            }
        }
        ProfScope ps(c, KC_GEMM_Q);
        DN_HIP(c, (launch_gemm<KC, KC, KC_GEMM_Q>(g, tile, 1, c->stream)));
        DN_HIP(c, ps.end());
    }
    // 2. the two passes over the Jacobian blocks
    if (fused) {
        ProfScope ps(c, KC_JV_JTV_FUSED);
        DN_HIP(c, ps.err);
        // up to 16 waves per work-group; with more than 16 strip slots (hidden widths above 4096 in total)
        // every wave keeps two strips, which the register budget allows for n_L <= 12
        const int waves = std::min(a.nwslots, 16);
        const dim3 grid(s), block(64 * waves);
        if (a.nwslots <= 16) {
            if (nL <= 4)       hipLaunchKernelGGL((jv_jtv_fused_kernel<4, 1>), grid, block, 0, c->stream, a);
            else if (nL <= 8)  hipLaunchKernelGGL((jv_jtv_fused_kernel<8, 1>), grid, block, 0, c->stream, a);
            else if (nL <= 12) hipLaunchKernelGGL((jv_jtv_fused_kernel<12, 1>), grid, block, 0, c->stream, a);
            else               hipLaunchKernelGGL((jv_jtv_fused_kernel<16, 1>), grid, block, 0, c->stream, a);
        } else {
            if (nL <= 4)       hipLaunchKernelGGL((jv_jtv_fused_kernel<4, 2>), grid, block, 0, c->stream, a);
            else if (nL <= 8)  hipLaunchKernelGGL((jv_jtv_fused_kernel<8, 2>), grid, block, 0, c->stream, a);
            else               hipLaunchKernelGGL((jv_jtv_fused_kernel<12, 2>), grid, block, 0, c->stream, a);
        }
        DN_HIP(c, hipGetLastError());
        DN_HIP(c, ps.end());
    } else {
        const long long slab = (long long)s * c->ldr;   // one layer's rows of R
        if (L >= 2) {
            // block L-1 applied as a dense product:  (sigma' * q^{L-1}) A^L^T, added to q^L (full) or
            // kept as r^{L-1} (per-layer)
            GemmGroup g;
            g.nprob = 1;
            GemmProblem& p = g.p[0];
            float* dst = bd ? c->fptr(c->o_R) + (long long)(L - 2) * slab : c->fptr(c->o_Q[L]);
            const long long lddst = bd ? c->ldr : c->ld[L];
            p = mk_problem(c->fptr(c->o_Q[L - 1]), c->ld[L - 1], c->fptr(c->o_AL), c->ld[L - 1], dst, lddst, s, nL,
                           c->dims[L - 1]);
            if (!bd) {
                p.add = dst;
                p.ldadd = lddst;
            }
            ProfScope ps(c, KC_GEMM_IMPLICIT);
            DN_HIP(c, ps.err);
            DN_HIP(c, (launch_gemm<KC, KC, KC_GEMM_IMPLICIT>(g, 64, 1, c->stream)));
            DN_HIP(c, ps.end());
        }
        TeamPlan tp;
        DN_HIP(c, plan_team(c, a, tp));
        if (tp.ok) {
            // one read of the stored blocks: teams of work-groups, see jv_jtv_team_kernel
            ProfScope ps(c, KC_JV_JTV_TEAM);
            DN_HIP(c, ps.err);
            DN_HIP(c, launch_team(c, tp));
            DN_HIP(c, ps.end());
        } else {
            {
                ProfScope ps(c, KC_JV);
                DN_HIP(c, ps.err);
                constexpr int UB = 16;
                hipLaunchKernelGGL(jv_rows_kernel<UB>, dim3(s * cdiv(nL, UB)), dim3(256), 0, c->stream, a);
                DN_HIP(c, hipGetLastError());
                DN_HIP(c, ps.end());
            }
            {
                ProfScope ps(c, KC_JTV);
                DN_HIP(c, ps.err);
                int chunks = 1;
                for (int m = 1; m + 1 < L; ++m) chunks += cdiv(c->dims[m], 1024);
                hipLaunchKernelGGL(jtv_cols_kernel, dim3((unsigned)((long long)s * chunks)), dim3(256),
                                   sizeof(float) * nL, c->stream, a, chunks);
                DN_HIP(c, hipGetLastError());
                DN_HIP(c, ps.end());
            }
        }
        if (L >= 2) {
            // t^{L-1} = sigma' * (A^L^T 2r):  T^L already holds 2r (full); per-layer uses 2 r^{L-1}
            GemmGroup g;
            g.nprob = 1;
            GemmProblem& p = g.p[0];
            const float* src = bd ? c->fptr(c->o_R) + (long long)(L - 2) * slab : c->fptr(c->o_T[L]);
            const long long ldsrc = bd ? c->ldr : c->ld[L];
            p = mk_problem(src, ldsrc, c->fptr(c->o_AL), c->ld[L - 1], c->fptr(c->o_T[L - 1]), c->ld[L - 1], s,
                           c->dims[L - 1], nL);
            p.aux = c->fptr(c->o_ZS[L - 1]);
            p.ldaux = c->ld[L - 1];
            p.alpha = bd ? 2.0f : 1.0f;
            ProfScope ps(c, KC_GEMM_IMPLICIT);
            DN_HIP(c, ps.err);
            DN_HIP(c, (launch_gemm<KC, RT, KC_GEMM_IMPLICIT>(g, 64, 1, c->stream)));
            DN_HIP(c, ps.end());
        }
    }
    // 3. sums over samples for every layer: W_m = T^m^T [Z^{m-1}, 1]
    TnPlan pl = plan_tn(c, s, true, 0);
    if (pl.total > c->tn_floats) return DN_ENOSPC;
    {
        GemmGroup g;
        g.nprob = L;
        for (int m = 1; m <= L; ++m) {
            GemmProblem& p = g.p[m - 1];
            p = mk_problem(c->fptr(c->o_T[m]), c->ld[m], c->fptr(c->o_ZS[m - 1]), c->ld[m - 1],
                           c->fptr(c->o_tn) + pl.offset[m], c->ldw[m], c->dims[m], c->dims[m - 1] + 1, s);
            p.b_ones_col = 1;
            p.split_stride = (long long)c->dims[m] * c->ldw[m];
        }
        ProfScope ps(c, KC_GEMM_TN_MATVEC);
        DN_HIP(c, ps.err);
        DN_HIP(c, (launch_gemm<RT, RT, KC_GEMM_TN_MATVEC>(g, pl.tile, pl.splits, c->stream)));
        DN_HIP(c, ps.end());
    }
    // 4. fold slices, scale by 1/|S|, add v/C
    return tn_reduce(c, &pl, false, v, out, 1.0 / (double)s);
}

void build_segs(const dn_ctx* c, int mode, CgSegs& sg) {
    std::memset(&sg, 0, sizeof(sg));
    if (mode == DN_PARTITION) {
        sg.nseg = c->nparts;
        for (int k = 0; k <= c->nparts; ++k) sg.off[k] = c->part_off[k];
    } else if (mode == DN_BLOCKDIAG) {
        sg.nseg = c->L;
        for (int m = 1; m <= c->L; ++m) sg.off[m - 1] = c->woff[m];
        sg.off[c->L] = c->n;
    } else {
        sg.nseg = 1;
        sg.off[0] = 0;
        sg.off[1] = c->n;
    }
    // chunk size: about 768 work-groups in total (3 per CU; every segment adds at most one more), at least
    // 2048 elements each
    long long chunk = std::max<long long>(2048, round_up((c->n + 767) / 768, 1024));
    for (;;) {
        long long tot = 0;
        for (int k = 0; k < sg.nseg; ++k) tot += (sg.off[k + 1] - sg.off[k] + chunk - 1) / chunk;
        if (tot <= DN_MAX_PARTIALS) break;
        chunk *= 2;
    }
    sg.chunk = (int)chunk;
    int b = 0;
    for (int k = 0; k < sg.nseg; ++k) {
        sg.cb[k] = b;
        b += (int)((sg.off[k + 1] - sg.off[k] + chunk - 1) / chunk);
    }
    sg.cb[sg.nseg] = b;
}

bool bad_mode(int mode) { return mode != DN_FULL && mode != DN_BLOCKDIAG && mode != DN_PARTITION; }

// Product over the partitions of the split structure (Section 3.1, Section 4.1)
int gn_matvec_part(dn_ctx* c, const float* v, float* out) {
    const int L = c->L, s = c->s_cur, nL = c->dims[L];
    PartArgs a;
    std::memset(&a, 0, sizeof(a));
    a.L = L; a.s = s; a.nL = nL;
    for (int m = 0; m <= L; ++m) {
        a.n[m] = c->dims[m];
        a.ld[m] = c->ld[m];
        a.split[m] = c->split[m];
        for (int k = 0; k <= DN_MAX_SPLIT; ++k) a.bound[m][k] = c->gbound[m][k];
    }
    for (int m = 1; m <= L + 1; ++m) a.part_base[m] = c->part_base[m];
    for (int m = 1; m < L; ++m) a.P[m] = c->fptr(c->o_P[m]);
    for (int m = 1; m <= L; ++m) {
        a.Qp[m] = c->fptr(c->o_Qp[m]);
        a.Tp[m] = c->fptr(c->o_Tp[m]);
    }
    a.R = c->fptr(c->o_Rp);
    a.ldr = c->ldr;
    // 1. inner sums over t, one product per (layer, input group); the bias term rides with group 0
    {
        GemmGroup g;
        g.nprob = 0;
        auto flush = [&]() -> int {
            if (g.nprob == 0) return DN_OK;
            ProfScope ps(c, KC_GEMM_Q);
            DN_HIP(c, ps.err);
            DN_HIP(c, (launch_gemm<KC, KC, KC_GEMM_Q>(g, 64, 1, c->stream)));
            DN_HIP(c, ps.end());
            g.nprob = 0;
            return DN_OK;
        };
        for (int m = 1; m <= L; ++m)
            for (int x = 0; x < c->split[m - 1]; ++x) {
                const int t0 = c->gbound[m - 1][x], t1 = c->gbound[m - 1][x + 1];
                GemmProblem& p = g.p[g.nprob++];
                p = mk_problem(c->fptr(c->o_ZS[m - 1]) + t0, c->ld[m - 1], v + c->woff[m] + t0, c->dims[m - 1],
                               c->fptr(c->o_Qp[m]) + (long long)x * s * c->ld[m], c->ld[m], s, c->dims[m], t1 - t0);
                if (x == 0) p.bias = v + c->boff[m];
                if (g.nprob == DN_MAX_GROUP) {
                    const int rc = flush();
                    if (rc != DN_OK) return rc;
                }
            }
        const int rc = flush();
        if (rc != DN_OK) return rc;
    }
    // 2. the passes over the stored blocks: one pass when a sample's strips fit one work-group's registers
    //    (as in the other modes), else the general two-pass kernels
    {
        int w = 0;
        for (int m = 1; m < L; ++m)
            for (int cidx = 0; cidx < cdiv(c->dims[m], 256); ++cidx, ++w)
                if (w < DN_MAX_WSLOTS) {
                    a.wlayer[w] = m;
                    a.wcol[w] = cidx;
                }
        a.nwslots = w;
    }
    const bool fused = L >= 2 && c->stream_passes != 2 &&
                       ((nL <= 16 && a.nwslots <= 16) || (nL <= 8 && a.nwslots <= DN_MAX_WSLOTS));
    if (fused) {
        ProfScope ps(c, KC_JV_JTV_FUSED);
        DN_HIP(c, ps.err);
        const dim3 grid(s), block(64 * std::min(a.nwslots, 16));
        if (a.nwslots <= 16) {
            if (nL <= 4)       hipLaunchKernelGGL((jv_jtv_fused_part_kernel<4, 1>), grid, block, 0, c->stream, a);
            else if (nL <= 8)  hipLaunchKernelGGL((jv_jtv_fused_part_kernel<8, 1>), grid, block, 0, c->stream, a);
            else if (nL <= 12) hipLaunchKernelGGL((jv_jtv_fused_part_kernel<12, 1>), grid, block, 0, c->stream, a);
            else               hipLaunchKernelGGL((jv_jtv_fused_part_kernel<16, 1>), grid, block, 0, c->stream, a);
        } else {
            if (nL <= 4)       hipLaunchKernelGGL((jv_jtv_fused_part_kernel<4, 2>), grid, block, 0, c->stream, a);
            else               hipLaunchKernelGGL((jv_jtv_fused_part_kernel<8, 2>), grid, block, 0, c->stream, a);
        }
        DN_HIP(c, hipGetLastError());
        DN_HIP(c, ps.end());
    } else {
        if (L >= 2) {
            ProfScope ps(c, KC_JV);
            DN_HIP(c, ps.err);
            hipLaunchKernelGGL(jv_part_kernel, dim3(s * cdiv(nL, 4)), dim3(256), 0, c->stream, a);
            DN_HIP(c, hipGetLastError());
            DN_HIP(c, ps.end());
        }
        ProfScope ps(c, KC_JTV);
        DN_HIP(c, ps.err);
        int chunks = 1;
        for (int m = 1; m < L; ++m) chunks += cdiv(c->dims[m], 256);
        int most = 1;
        for (int m = 1; m < L; ++m) most = std::max(most, c->split[m - 1] * c->split[m]);
        const size_t lds = sizeof(float) * (size_t)most * nL;
        hipLaunchKernelGGL(jtv_part_kernel, dim3((unsigned)((long long)s * chunks)), dim3(256), lds, c->stream, a,
                           chunks);
        DN_HIP(c, hipGetLastError());
        DN_HIP(c, ps.end());
    }
    // 3. sums over samples, one product per (layer, input group) into that group's columns; bias sums apart
    TnPlan pl = plan_tn(c, s, true, 0);
    if (pl.total > c->tn_floats) return DN_ENOSPC;
    {
        GemmGroup g;
        g.nprob = 0;
        auto flush = [&]() -> int {
            if (g.nprob == 0) return DN_OK;
            ProfScope ps(c, KC_GEMM_TN_MATVEC);
            DN_HIP(c, ps.err);
            DN_HIP(c, (launch_gemm<RT, RT, KC_GEMM_TN_MATVEC>(g, pl.tile, pl.splits, c->stream)));
            DN_HIP(c, ps.end());
            g.nprob = 0;
            return DN_OK;
        };
        for (int m = 1; m <= L; ++m)
            for (int x = 0; x < c->split[m - 1]; ++x) {
                const int t0 = c->gbound[m - 1][x], t1 = c->gbound[m - 1][x + 1];
                GemmProblem& p = g.p[g.nprob++];
                p = mk_problem(c->fptr(c->o_Tp[m]) + (long long)x * s * c->ld[m], c->ld[m], c->fptr(c->o_ZS[m - 1]) + t0,
                               c->ld[m - 1], c->fptr(c->o_tn) + pl.offset[m] + t0, c->ldw[m], c->dims[m], t1 - t0, s);
                p.split_stride = (long long)c->dims[m] * c->ldw[m];
                if (g.nprob == DN_MAX_GROUP) {
                    const int rc = flush();
                    if (rc != DN_OK) return rc;
                }
            }
        const int rc = flush();
        if (rc != DN_OK) return rc;
        BiasSumArgs ba;
        std::memset(&ba, 0, sizeof(ba));
        ba.L = L; ba.s = s; ba.splits = pl.splits;
        // the K-slices are those of the products above (finalize_group: slice length rounded up to the K tile)
        ba.k_per_split = (int)round_up(cdiv(s, pl.splits), 16);
        int chunks = 0;
        for (int m = 0; m <= L; ++m) { ba.n[m] = c->dims[m]; ba.ld[m] = c->ld[m]; }
        for (int m = 1; m <= L; ++m) {
            ba.T0[m] = c->fptr(c->o_Tp[m]);
            ba.W[m] = c->fptr(c->o_tn) + pl.offset[m];
            ba.ldw[m] = c->ldw[m];
            ba.first[m] = chunks;
            chunks += cdiv(c->dims[m], 16);
        }
        ba.first[L + 1] = chunks;
        ProfScope ps(c, KC_TN_REDUCE);
        DN_HIP(c, ps.err);
        hipLaunchKernelGGL(bias_colsum_kernel, dim3(chunks * pl.splits), dim3(256), 0, c->stream, ba);
        DN_HIP(c, hipGetLastError());
        DN_HIP(c, ps.end());
    }
    // 4. fold slices, scale by 1/|S|, add v/C
    return tn_reduce(c, &pl, false, v, out, 1.0 / (double)s);
}

}  // namespace

// ================================================================================================
extern "C" {

const char* dn_strerror(int code) {
    switch (code) {
        case DN_OK: return "ok";
        case DN_EINVAL: return "invalid argument";
        case DN_ENOSPC: return "workspace too small";
        case DN_ESTATE: return "call out of order (no workspace bound, or no Jacobian prepared)";
        case DN_EHIP: return "HIP runtime error";
        case DN_ENOMEM: return "host allocation failed";
        case DN_ETIMEOUT: return "a bounded wait between work-groups ran out";
        default: return "unknown error code";
    }
}

int dn_create(dn_ctx** out, int L, const int* dims, double C, int l_max, int s_max) {
    if (!out) return DN_EINVAL;
    *out = nullptr;
    if (!dims || L < 1 || L > DN_MAX_LAYERS || !(C > 0.0) || l_max < 1 || s_max < 1) return DN_EINVAL;
    for (int m = 0; m <= L; ++m)
        if (dims[m] < 1) return DN_EINVAL;
    // row counts of the batched sweeps are int: s_max * n_L rows
    if ((long long)s_max * dims[L] > 0x7fffffffLL) return DN_EINVAL;
    dn_ctx* c = new (std::nothrow) dn_ctx();
    if (!c) return DN_ENOMEM;
    c->L = L;
    c->C = C;
    c->l_max = l_max;
    c->s_max = s_max;
    long long o = 0;
    for (int m = 0; m <= L; ++m) {
        c->dims[m] = dims[m];
        c->ld[m] = round_up(dims[m], 4);
        if (m >= 1) {
            c->woff[m] = o;
            o += (long long)dims[m - 1] * dims[m];
            c->boff[m] = o;
            o += dims[m];
            c->ldw[m] = round_up(dims[m - 1] + 1, 4);
        }
    }
    c->n = o;
    c->ldr = round_up(dims[L], 4);
    layout_workspace(c);
    *out = c;
    return DN_OK;
}

void dn_destroy(dn_ctx* c) {
    if (!c) return;
    for (auto& p : c->pending) {
        (void)hipEventDestroy(p.a);
        (void)hipEventDestroy(p.b);
    }
    for (auto e : c->free_events) (void)hipEventDestroy(e);
    delete c;
}

size_t dn_num_params(const dn_ctx* c) { return c ? (size_t)c->n : 0; }
size_t dn_workspace_bytes(const dn_ctx* c) { return c ? c->ws_bytes : 0; }
int dn_last_hip_error(const dn_ctx* c) { return c ? c->last_hip : 0; }

int dn_bind(dn_ctx* c, void* d_workspace, size_t bytes, void* hip_stream) {
    if (!c || !d_workspace) return DN_EINVAL;
    if ((reinterpret_cast<uintptr_t>(d_workspace) & 255u) != 0) return DN_EINVAL;
    if (bytes < c->ws_bytes) return DN_ENOSPC;
    c->ws = static_cast<char*>(d_workspace);
    c->stream = static_cast<hipStream_t>(hip_stream);
    c->bound = true;
    c->prepped = false;
    c->team_clean = false;
    c->team_used = false;
    c->split_set = false;
    // size of the chip, for kernels whose grid must be resident all at once (default kept if no device answers)
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) == hipSuccess &&
        hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && cus > 0)
        c->num_cus = cus;
    else
        (void)hipGetLastError();
    return DN_OK;
}

int dn_forward(dn_ctx* c, const float* theta, const float* X, const float* Y, int l, double* f_host, float* ZL) {
    if (!c || !theta || !X || !Y || !f_host || l < 1) return DN_EINVAL;
    if (!c->bound) return DN_ESTATE;
    const int L = c->L, n0 = c->dims[0], nL = c->dims[L];
    // the samples go through in chunks of at most l_max rows that reuse the same activation buffers
    for (int r0 = 0; r0 < l; r0 += c->l_max) {
        const int rows = std::min(c->l_max, l - r0);
        int rc = forward_layers(c, theta, X + (long long)r0 * n0, n0, rows, c->o_Zall, L);
        if (rc != DN_OK) return rc;
        rc = objective(c, theta, Y + (long long)r0 * nL, rows, l, r0 == 0, r0 + rows == l, nullptr, 0,
                       ZL ? ZL + (long long)r0 * nL : nullptr, f_host);
        if (rc != DN_OK) return rc;
    }
    return DN_OK;
}

int dn_grad(dn_ctx* c, const float* theta, const float* X, const float* Y, int l, float* g, double* f_host) {
    if (!c || !theta || !X || !Y || !g || l < 1) return DN_EINVAL;
    if (!c->bound) return DN_ESTATE;
    const int L = c->L, n0 = c->dims[0], nL = c->dims[L];
    if (L >= 2) {
        int rc = transpose_weights(c, theta, 2, L);
        if (rc != DN_OK) return rc;
    }
    // plan of the sums over samples, from the size of a full chunk; every chunk adds into the same slices
    const int rows_full = std::min(l, c->l_max);
    TnPlan plans[DN_MAX_LAYERS + 1];
    // partial buffers of different layers must not overlap: give each layer its own range
    long long tn_off = 0;
    for (int m = 1; m <= L; ++m) {
        plans[m] = plan_tn(c, rows_full, false, m);
        plans[m].offset[m] = tn_off;
        tn_off += round_up(plans[m].floats[m], 64);
    }
    if (tn_off > c->tn_floats) {
        // fall back to one slice per layer, which always fits
        tn_off = 0;
        for (int m = 1; m <= L; ++m) {
            plans[m].splits = 1;
            plans[m].k_per_split = (int)round_up(rows_full, kBKmax);
            plans[m].floats[m] = (long long)c->dims[m] * c->ldw[m];
            plans[m].offset[m] = tn_off;
            tn_off += round_up(plans[m].floats[m], 64);
        }
        if (tn_off > c->tn_floats) return DN_ENOSPC;
    }
    for (int r0 = 0; r0 < l; r0 += c->l_max) {
        const int rows = std::min(c->l_max, l - r0);
        const float* Xc = X + (long long)r0 * n0;
        int rc = forward_layers(c, theta, Xc, n0, rows, c->o_Zall, L);
        if (rc != DN_OK) return rc;
        // seed 2 (z^L - y) into D[0]
        int cur = 0;
        rc = objective(c, theta, Y + (long long)r0 * nL, rows, l, r0 == 0, r0 + rows == l, c->fptr(c->o_D[cur]),
                       c->ld[L], nullptr, f_host);
        if (rc != DN_OK) return rc;
        for (int m = L; m >= 1; --m) {
            const float* delta = c->fptr(c->o_D[cur]);
            const float* zprev = (m == 1) ? Xc : c->fptr(c->o_Zall[m - 1]);
            const long long ldprev = (m == 1) ? n0 : c->ld[m - 1];
            {
                // sum over samples: delta^m^T [z^{m-1}, 1]
                GemmGroup g1;
                g1.nprob = 1;
                GemmProblem& p = g1.p[0];
                p = mk_problem(delta, c->ld[m], zprev, ldprev, c->fptr(c->o_tn) + plans[m].offset[m], c->ldw[m],
                               c->dims[m], c->dims[m - 1] + 1, rows);
                p.b_ones_col = 1;
                p.split_stride = (long long)c->dims[m] * c->ldw[m];
                p.accumulate = r0 > 0 ? 1 : 0;
                ProfScope ps(c, KC_GEMM_TN_GRAD);
                DN_HIP(c, ps.err);
                DN_HIP(c, (launch_gemm<RT, RT, KC_GEMM_TN_GRAD>(g1, plans[m].tile, plans[m].splits, c->stream)));
                DN_HIP(c, ps.end());
            }
            if (m > 1) {
                // delta^{m-1} = (delta^m (W^m)^T) * z^{m-1} (1 - z^{m-1})
                GemmGroup g2;
                g2.nprob = 1;
                GemmProblem& p = g2.p[0];
                p = mk_problem(delta, c->ld[m], c->fptr(c->o_WT) + c->woff[m], c->dims[m], c->fptr(c->o_D[cur ^ 1]),
                               c->ld[m - 1], rows, c->dims[m - 1], c->dims[m]);
                p.aux = zprev;
                p.ldaux = ldprev;
                p.auxdiv = 1;
                const int tile = pick_tile(g2, true);
                ProfScope ps(c, KC_GEMM_BACK);
                DN_HIP(c, ps.err);
                DN_HIP(c, (launch_gemm<KC, KC, KC_GEMM_BACK>(g2, tile, 1, c->stream)));
                DN_HIP(c, ps.end());
                cur ^= 1;
            }
        }
    }
    return tn_reduce(c, plans, true, theta, g, 1.0 / (double)l);
}

int dn_jacobian_prep(dn_ctx* c, const float* theta, const float* X, int l, const int* S, int s) {
    if (!c || !theta || !X || !S || l < 1 || s < 1 || s > c->s_max) return DN_EINVAL;
    if (!c->bound) return DN_ESTATE;
    const int L = c->L, nL = c->dims[L];
    c->prepped = false;
    {
        ProfScope ps(c, KC_GATHER);
        DN_HIP(c, ps.err);
        hipLaunchKernelGGL(gather_rows_kernel, dim3(grid_for((long long)s * c->dims[0])), dim3(256), 0, c->stream, X,
                           S, c->fptr(c->o_ZS[0]), s, c->dims[0], l, (long long)c->dims[0], c->ld[0]);
        DN_HIP(c, hipGetLastError());
        DN_HIP(c, ps.end());
    }
    // z^{m,i} for the hidden layers (the output layer's activations are not needed by the products)
    int rc = forward_layers(c, theta, c->fptr(c->o_ZS[0]), c->ld[0], s, c->o_ZS, L - 1);
    if (rc != DN_OK) return rc;
    if (L >= 2) {
        ProfScope ps(c, KC_JAC_INIT);
        DN_HIP(c, ps.err);
        // keep a copy of A^L: the products rebuild block L-1 from it
        hipLaunchKernelGGL(pad_rows_kernel, dim3(grid_for((long long)nL * c->dims[L - 1])), dim3(256), 0, c->stream,
                           theta + c->woff[L], c->fptr(c->o_AL), (long long)nL, c->dims[L - 1], c->ld[L - 1]);
        DN_HIP(c, hipGetLastError());
        const dim3 jgrid(std::min(64, grid_for((long long)nL * c->ld[L - 1] / 4, 256)), std::min(s, 32768));
        hipLaunchKernelGGL(jac_init_kernel, jgrid, dim3(256), 0, c->stream, c->fptr(c->o_AL),
                           c->fptr(c->o_ZS[L - 1]), c->fptr(c->o_P[L - 1]), s, nL, c->dims[L - 1], c->ld[L - 1]);
        DN_HIP(c, hipGetLastError());
        DN_HIP(c, ps.end());
    }
    if (L >= 2) {
        rc = transpose_weights(c, theta, 2, L);
        if (rc != DN_OK) return rc;
    }
    DN_HIP(c, hipMemcpyAsync(c->fptr(c->o_thS), theta, sizeof(float) * (size_t)c->n, hipMemcpyDeviceToDevice, c->stream));
    // P^{m-1} = (P^m (W^m)^T) * sigma'(s^{m-1}):  the n_L backward sweeps of all samples as one product
    for (int m = L - 1; m >= 2; --m) {
        GemmGroup g;
        g.nprob = 1;
        GemmProblem& p = g.p[0];
        p = mk_problem(c->fptr(c->o_P[m]), c->ld[m], c->fptr(c->o_WT) + c->woff[m], c->dims[m], c->fptr(c->o_P[m - 1]),
                       c->ld[m - 1], s * nL, c->dims[m - 1], c->dims[m]);
        p.aux = c->fptr(c->o_ZS[m - 1]);
        p.ldaux = c->ld[m - 1];
        p.auxdiv = nL;
        const int tile = pick_tile(g, true);
        ProfScope ps(c, KC_GEMM_PREP);
        DN_HIP(c, ps.err);
        DN_HIP(c, (launch_gemm<KC, KC, KC_GEMM_PREP>(g, tile, 1, c->stream)));
        DN_HIP(c, ps.end());
    }
    c->s_cur = s;
    c->prepped = true;
    return DN_OK;
}

int dn_jacobian_read(dn_ctx* c, int m, float* P_out) {
    if (!c || !P_out || m < 1 || m >= c->L) return DN_EINVAL;
    if (!c->bound || !c->prepped) return DN_ESTATE;
    const long long rows = (long long)c->s_cur * c->dims[c->L];
    hipLaunchKernelGGL(unpad_rows_kernel, dim3(grid_for(rows * c->dims[m])), dim3(256), 0, c->stream,
                       c->fptr(c->o_P[m]), P_out, rows, c->dims[m], c->ld[m]);
    DN_HIP(c, hipGetLastError());
    return DN_OK;
}

int dn_gn_matvec(dn_ctx* c, const float* v, float* out, int mode) {
    if (!c || !v || !out || bad_mode(mode)) return DN_EINVAL;
    if (!c->bound || !c->prepped) return DN_ESTATE;
    return gn_matvec(c, v, out, mode);
}

namespace {
// CG of dn_cg / dn_cg_sync; r_percent <= 0 switches the joint termination of Section 4.4 off
int cg_run(dn_ctx* c, const float* g, double lambda, double sigma, int max_iter, int mode, int cg_min, double r_percent,
           float* d, int* iters_host, double* resnorm_host) {
    if (mode == DN_PARTITION && !c->split_set) return DN_ESTATE;
    CgSegs sg;
    build_segs(c, mode, sg);
    const int grid = sg.cb[sg.nseg];
    // With a split structure the CG vectors live in partition-major order (every partition contiguous, see
    // dn_set_split); the product takes and returns theta-layout vectors, so p is scattered before and q
    // gathered after every product.
    const bool part = mode == DN_PARTITION;
    const int* perm = reinterpret_cast<const int*>(c->ws + c->o_perm);
    const int vgrid = grid_for(c->n);
    float* d_cg = part ? c->fptr(c->o_dperm) : d;
    const float* g_cg = g;
    if (part) {
        hipLaunchKernelGGL(perm_gather_kernel, dim3(vgrid), dim3(256), 0, c->stream, g, perm, c->fptr(c->o_gperm), c->n,
                           1.0f);
        DN_HIP(c, hipGetLastError());
        g_cg = c->fptr(c->o_gperm);
    }
    float* r = c->fptr(c->o_r);
    float* p = c->fptr(c->o_p);
    float* q = c->fptr(c->o_q);
    double* part0 = c->dptr(c->o_part[0]);
    double* part1 = c->dptr(c->o_part[1]);
    double* part2 = c->dptr(c->o_part[2]);
    CgState* st = reinterpret_cast<CgState*>(c->ws + c->o_state);
    CgState hst;
    {
        ProfScope ps(c, KC_CG_VEC);
        DN_HIP(c, ps.err);
        hipLaunchKernelGGL(cg_init_kernel, dim3(grid), dim3(256), 0, c->stream, sg, g_cg, d_cg, r, p, part0);
        DN_HIP(c, hipGetLastError());
        hipLaunchKernelGGL(cg_init_state_kernel, dim3(1), dim3(256), 0, c->stream, sg, part0, st);
        DN_HIP(c, hipGetLastError());
        DN_HIP(c, ps.end());
    }
    DN_HIP(c, hipMemcpyAsync(&hst, st, sizeof(CgState), hipMemcpyDeviceToHost, c->stream));
    DN_HIP(c, hipStreamSynchronize(c->stream));
    auto any_active = [&](const CgState& s) {
        for (int k = 0; k < sg.nseg; ++k)
            if (s.active[k]) return true;
        return false;
    };
    const bool joint = r_percent > 0.0;
    auto joint_stop = [&](const CgState& s, int k) {
        int finished = 0;
        for (int b = 0; b < sg.nseg; ++b) finished += s.active[b] ? 0 : 1;
        return k >= cg_min && (double)finished >= r_percent / 100.0 * (double)sg.nseg;
    };
    int iters = 0;
    bool active = any_active(hst);
    while (iters < max_iter && active) {
        int rc;
        if (part) {
            hipLaunchKernelGGL(perm_scatter_kernel, dim3(vgrid), dim3(256), 0, c->stream, p, perm, c->fptr(c->o_ptheta),
                               c->n);
            DN_HIP(c, hipGetLastError());
            rc = gn_matvec(c, c->fptr(c->o_ptheta), c->fptr(c->o_qtheta), mode);
            if (rc != DN_OK) return rc;
            hipLaunchKernelGGL(perm_gather_kernel, dim3(vgrid), dim3(256), 0, c->stream, c->fptr(c->o_qtheta), perm, q,
                               c->n, 1.0f);
            DN_HIP(c, hipGetLastError());
        } else {
            rc = gn_matvec(c, p, q, mode);
            if (rc != DN_OK) return rc;
        }
        const CgState* cur = st + (iters & 1);
        CgState* nxt = st + ((iters + 1) & 1);
        {
            ProfScope ps(c, KC_CG_VEC);
            DN_HIP(c, ps.err);
            hipLaunchKernelGGL(cg_dot_kernel, dim3(grid), dim3(256), 0, c->stream, sg, p, q, (float)lambda, part1);
            DN_HIP(c, hipGetLastError());
            hipLaunchKernelGGL(cg_update_dr_kernel, dim3(grid), dim3(256), 0, c->stream, sg, cur, part1, p, q,
                               (float)lambda, d_cg, r, part2);
            DN_HIP(c, hipGetLastError());
            hipLaunchKernelGGL(cg_update_p_kernel, dim3(grid), dim3(256), 0, c->stream, sg, cur, nxt, part2,
                               sigma * sigma, r, p);
            DN_HIP(c, hipGetLastError());
            DN_HIP(c, ps.end());
        }
        ++iters;
        if (sigma > 0.0) {
            DN_HIP(c, hipMemcpyAsync(&hst, nxt, sizeof(CgState), hipMemcpyDeviceToHost, c->stream));
            DN_HIP(c, hipStreamSynchronize(c->stream));
            active = any_active(hst);
            if (joint && joint_stop(hst, iters)) break;
        }
    }
    if (part) {
        hipLaunchKernelGGL(perm_scatter_kernel, dim3(vgrid), dim3(256), 0, c->stream, d_cg, perm, d, c->n);
        DN_HIP(c, hipGetLastError());
    }
    DN_HIP(c, hipMemcpyAsync(&hst, st + (iters & 1), sizeof(CgState), hipMemcpyDeviceToHost, c->stream));
    DN_HIP(c, hipStreamSynchronize(c->stream));
    *iters_host = iters;
    for (int k = 0; k < sg.nseg; ++k) resnorm_host[k] = std::sqrt(hst.rho[k]);
    return team_status(c);
}
}  // namespace

int dn_cg(dn_ctx* c, const float* g, double lambda, double sigma, int max_iter, int mode, float* d, int* iters_host,
          double* resnorm_host) {
    if (!c || !g || !d || !iters_host || !resnorm_host || bad_mode(mode) || max_iter < 1 || !(lambda >= 0.0) ||
        !(sigma >= 0.0))
        return DN_EINVAL;
    if (!c->bound || !c->prepped) return DN_ESTATE;
    return cg_run(c, g, lambda, sigma, max_iter, mode, 0, 0.0, d, iters_host, resnorm_host);
}

int dn_cg_sync(dn_ctx* c, const float* g, double lambda, double sigma, int max_iter, int mode, int cg_min,
               double r_percent, float* d, int* iters_host, double* resnorm_host) {
    if (!c || !g || !d || !iters_host || !resnorm_host || max_iter < 1 || cg_min < 0 || !(lambda >= 0.0) ||
        !(sigma >= 0.0) || !(r_percent > 0.0 && r_percent <= 100.0) || (mode != DN_BLOCKDIAG && mode != DN_PARTITION))
        return DN_EINVAL;
    if (!c->bound || !c->prepped) return DN_ESTATE;
    return cg_run(c, g, lambda, sigma, max_iter, mode, cg_min, r_percent, d, iters_host, resnorm_host);
}

int dn_num_partitions(const dn_ctx* c) { return (c && c->split_set) ? c->nparts : 0; }

int dn_set_split(dn_ctx* c, const int* groups) {
    if (!c || !groups) return DN_EINVAL;
    const int L = c->L;
    for (int m = 0; m <= L; ++m)
        if (groups[m] < 1 || groups[m] > DN_MAX_SPLIT || groups[m] > c->dims[m]) return DN_EINVAL;
    if (!c->bound) return DN_ESTATE;
    c->split_set = false;
    int np = 0;
    for (int m = 0; m <= L; ++m) {
        c->split[m] = groups[m];
        for (int k = 0; k <= DN_MAX_SPLIT; ++k)
            c->gbound[m][k] = (int)((long long)std::min(k, groups[m]) * c->dims[m] / groups[m]);
        if (m >= 1) {
            c->part_base[m] = np;
            np += groups[m - 1] * groups[m];
        }
    }
    c->part_base[L + 1] = np;
    c->nparts = np;
    // index map: theta indices partition by partition (layer, input group a, output group b; inside a
    // partition the weights row by row, then the biases for a = 0)
    std::vector<int> perm;
    try {
        perm.resize((size_t)c->n);
    } catch (const std::bad_alloc&) {
        return DN_ENOMEM;
    }
    long long k = 0;
    int pid = 0;
    for (int m = 1; m <= L; ++m) {
        const int nprev = c->dims[m - 1];
        for (int a = 0; a < groups[m - 1]; ++a)
            for (int b = 0; b < groups[m]; ++b) {
                c->part_off[pid++] = k;
                for (int j = c->gbound[m][b]; j < c->gbound[m][b + 1]; ++j)
                    for (int t = c->gbound[m - 1][a]; t < c->gbound[m - 1][a + 1]; ++t)
                        perm[(size_t)k++] = (int)(c->woff[m] + (long long)j * nprev + t);
                if (a == 0)
                    for (int j = c->gbound[m][b]; j < c->gbound[m][b + 1]; ++j) perm[(size_t)k++] = (int)(c->boff[m] + j);
            }
    }
    c->part_off[pid] = k;
    if (k != c->n) return DN_EINVAL;
    DN_HIP(c, hipMemcpyAsync(c->ws + c->o_perm, perm.data(), sizeof(int) * (size_t)c->n, hipMemcpyHostToDevice,
                             c->stream));
    DN_HIP(c, hipStreamSynchronize(c->stream));
    c->split_set = true;
    return DN_OK;
}

int dn_newton_step(dn_ctx* c, float* theta, const float* X, const float* Y, int l, const int* S, int s, float* d_prev,
                   dn_newton_params* prm, dn_newton_stats* st) {
    if (!c || !theta || !X || !Y || !S || !d_prev || !prm || !st || l < 1 || s < 1 || s > c->s_max)
        return DN_EINVAL;
    if (bad_mode(prm->mode) || prm->cg_max < 1 || prm->max_trials < 1 || !(prm->lambda >= 0.0) ||
        !(prm->sigma >= 0.0) || !(prm->eta > 0.0 && prm->eta < 1.0) || !(prm->drop > 0.0 && prm->drop <= 1.0) ||
        !(prm->boost >= 1.0) || prm->cg_min < 0 || !(prm->r_percent <= 100.0))
        return DN_EINVAL;
    if (!c->bound) return DN_ESTATE;
    std::memset(st, 0, sizeof(*st));
    const long long n = c->n;
    float* g = c->fptr(c->o_ng);
    float* d = c->fptr(c->o_nd);
    float* Gd = c->fptr(c->o_nGd);
    float* Gdb = c->fptr(c->o_nGdb);
    float* trial = c->fptr(c->o_ntheta);
    double* part = c->dptr(c->o_npart);
    double* dots_dev = c->dptr(c->o_f) + 8;
    const int vgrid = grid_for(n);
    const int dgrid = std::min(DN_MAX_PARTIALS, vgrid);

    // 1-3: gradient on all rows, Jacobian blocks on S, CG direction
    double f0 = 0.0;
    int rc = dn_grad(c, theta, X, Y, l, g, &f0);
    if (rc != DN_OK) return rc;
    rc = dn_jacobian_prep(c, theta, X, l, S, s);
    if (rc != DN_OK) return rc;
    double resn[DN_MAX_SEGS];
    const bool joint = prm->mode != DN_FULL && prm->r_percent > 0.0;
    rc = cg_run(c, g, prm->lambda, prm->sigma, prm->cg_max, prm->mode, joint ? prm->cg_min : 0,
                joint ? prm->r_percent : 0.0, d, &st->cg_iters, resn);
    if (rc != DN_OK) return rc;

    // 4: inner products with the whole G^S
    rc = gn_matvec(c, d, Gd, DN_FULL);
    if (rc != DN_OK) return rc;
    const float* db = prm->combine ? d_prev : d;        // without combination the d_prev slots repeat d
    if (prm->combine) {
        rc = gn_matvec(c, d_prev, Gdb, DN_FULL);
        if (rc != DN_OK) return rc;
    }
    double dots[5];
    {
        ProfScope ps(c, KC_CG_VEC);
        DN_HIP(c, ps.err);
        hipLaunchKernelGGL(newton_dots_kernel, dim3(dgrid), dim3(256), 0, c->stream, g, d, db, Gd,
                           prm->combine ? Gdb : Gd, n, part);
        DN_HIP(c, hipGetLastError());
        hipLaunchKernelGGL(newton_dots_finalize_kernel, dim3(1), dim3(256), 0, c->stream, part, dgrid, dots_dev);
        DN_HIP(c, hipGetLastError());
        DN_HIP(c, ps.end());
    }
    DN_HIP(c, hipMemcpyAsync(dots, dots_dev, sizeof(dots), hipMemcpyDeviceToHost, c->stream));
    DN_HIP(c, hipStreamSynchronize(c->stream));
    double beta1 = 1.0, beta2 = 0.0;
    const double a11 = dots[2], a12 = dots[3], a22 = dots[4];
    if (prm->combine) {
        const double b1 = -dots[0], b2 = -dots[1];
        const double det = a11 * a22 - a12 * a12;
        if (det > prm->eps) {
            beta1 = (b1 * a22 - b2 * a12) / det;
            beta2 = (a11 * b2 - a12 * b1) / det;
        }
    }
    double gTd = dots[0], dGd = a11;
    if (beta1 != 1.0 || beta2 != 0.0) {
        ProfScope ps(c, KC_CG_VEC);
        DN_HIP(c, ps.err);
        hipLaunchKernelGGL(axpby_kernel, dim3(vgrid), dim3(256), 0, c->stream, (float)beta1, d, (float)beta2, d_prev,
                           d, n);
        DN_HIP(c, hipGetLastError());
        DN_HIP(c, ps.end());
        gTd = beta1 * dots[0] + beta2 * dots[1];
        dGd = beta1 * beta1 * a11 + 2.0 * beta1 * beta2 * a12 + beta2 * beta2 * a22;
    }
    st->beta1 = beta1; st->beta2 = beta2; st->gTd = gTd; st->dGd = dGd; st->f_old = f0;

    // 5: backtracking line search on f
    double alpha = 1.0, f_new = f0;
    bool accepted = false;
    for (int k = 0; k < prm->max_trials; ++k) {
        {
            ProfScope ps(c, KC_CG_VEC);
            DN_HIP(c, ps.err);
            hipLaunchKernelGGL(axpby_kernel, dim3(vgrid), dim3(256), 0, c->stream, 1.0f, theta, (float)alpha, d, trial,
                               n);
            DN_HIP(c, hipGetLastError());
            DN_HIP(c, ps.end());
        }
        double f_try = 0.0;
        rc = dn_forward(c, trial, X, Y, l, &f_try, nullptr);
        if (rc != DN_OK) return rc;
        st->f_evals = k + 1;
        if (f_try <= f0 + prm->eta * alpha * gTd) {
            f_new = f_try;
            accepted = true;
            break;
        }
        alpha *= 0.5;
    }
    // 6: ratio of actual to predicted reduction, next lambda; advance theta, remember the direction
    if (accepted) {
        st->alpha = alpha;
        st->rho = (f_new - f0) / (alpha * gTd + 0.5 * alpha * alpha * dGd);
        if (st->rho > 0.75) prm->lambda *= prm->drop;
        else if (!(st->rho >= 0.25)) prm->lambda *= prm->boost;
        DN_HIP(c, hipMemcpyAsync(theta, trial, sizeof(float) * (size_t)n, hipMemcpyDeviceToDevice, c->stream));
    } else {
        st->alpha = 0.0;
        st->rho = 0.0;
        prm->lambda *= prm->boost;
    }
    st->f_new = f_new;
    DN_HIP(c, hipMemcpyAsync(d_prev, d, sizeof(float) * (size_t)n, hipMemcpyDeviceToDevice, c->stream));
    DN_HIP(c, hipStreamSynchronize(c->stream));
    return team_status(c);
}

int dn_set_stream_passes(dn_ctx* c, int passes) {
    if (!c || (passes != 0 && passes != 2)) return DN_EINVAL;
    c->stream_passes = passes;
    return DN_OK;
}

int dn_set_spin_limit(dn_ctx* c, unsigned polls) {
    if (!c) return DN_EINVAL;
    c->spin_limit = polls;
    return DN_OK;
}

int dn_sync_status(dn_ctx* c) {
    if (!c) return DN_EINVAL;
    if (!c->bound) return DN_ESTATE;
    DN_HIP(c, hipStreamSynchronize(c->stream));
    return team_status(c);
}

int dn_gn_matvec_rop(dn_ctx* c, const float* v, float* out) {
    if (!c || !v || !out) return DN_EINVAL;
    if (!c->bound || !c->prepped) return DN_ESTATE;
    const int L = c->L, s = c->s_cur;
    const float* th = c->fptr(c->o_thS);
    // 1. inner sums over t for every layer, Q^m = Z^{m-1} V^m + vb^m; layer 1's result is at once the
    //    derivative of z^1 along v:  zdot^1 = sigma'(s^1) * Q^1
    {
        GemmGroup g;
        g.nprob = L;
        for (int m = 1; m <= L; ++m) {
            g.p[m - 1] = mk_problem(c->fptr(c->o_ZS[m - 1]), c->ld[m - 1], v + c->woff[m], c->dims[m - 1],
                                    c->fptr(c->o_Q[m]), c->ld[m], s, c->dims[m], c->dims[m - 1]);
            g.p[m - 1].bias = v + c->boff[m];
        }
        if (L >= 2) {
            g.p[0].aux = c->fptr(c->o_ZS[1]);
            g.p[0].ldaux = c->ld[1];
        }
        const int tile = pick_tile(g, true);
        ProfScope ps(c, KC_GEMM_Q);
        DN_HIP(c, ps.err);
        DN_HIP(c, (launch_gemm<KC, KC, KC_GEMM_Q>(g, tile, 1, c->stream)));
        DN_HIP(c, ps.end());
    }
    // 2. forward sweep of the derivative: zdot^m = sigma'(s^m) * (Q^m + zdot^{m-1} W^m), in place in Q^m;
    //    at the output layer sigma' = 1 and Q^L becomes J^i v
    for (int m = 2; m <= L; ++m) {
        GemmGroup g;
        g.nprob = 1;
        GemmProblem& p = g.p[0];
        p = mk_problem(c->fptr(c->o_Q[m - 1]), c->ld[m - 1], th + c->woff[m], c->dims[m - 1], c->fptr(c->o_Q[m]),
                       c->ld[m], s, c->dims[m], c->dims[m - 1]);
        p.pre = c->fptr(c->o_Q[m]);
        p.ldpre = c->ld[m];
        if (m < L) {
            p.aux = c->fptr(c->o_ZS[m]);
            p.ldaux = c->ld[m];
        }
        const int tile = pick_tile(g, true);
        ProfScope ps(c, KC_GEMM_ROP);
        DN_HIP(c, ps.err);
        DN_HIP(c, (launch_gemm<KC, KC, KC_GEMM_ROP>(g, tile, 1, c->stream)));
        DN_HIP(c, ps.end());
    }
    // 3. back-propagation with seed J^i v (the factor 2 of B = 2I goes into the final scale):
    //    delta^L = Q^L,  delta^{m-1} = (delta^m (W^m)^T) * sigma'(s^{m-1})  ->  T^{m-1}
    for (int m = L; m >= 2; --m) {
        GemmGroup g;
        g.nprob = 1;
        GemmProblem& p = g.p[0];
        const float* delta = m == L ? c->fptr(c->o_Q[L]) : c->fptr(c->o_T[m]);
        p = mk_problem(delta, c->ld[m], c->fptr(c->o_WT) + c->woff[m], c->dims[m], c->fptr(c->o_T[m - 1]), c->ld[m - 1], s,
                       c->dims[m - 1], c->dims[m]);
        p.aux = c->fptr(c->o_ZS[m - 1]);
        p.ldaux = c->ld[m - 1];
        const int tile = pick_tile(g, true);
        ProfScope ps(c, KC_GEMM_ROP);
        DN_HIP(c, ps.err);
        DN_HIP(c, (launch_gemm<KC, KC, KC_GEMM_ROP>(g, tile, 1, c->stream)));
        DN_HIP(c, ps.end());
    }
    // 4. sums over samples for every layer, then out = v/C + (2/|S|) * sums
    TnPlan pl = plan_tn(c, s, true, 0);
    if (pl.total > c->tn_floats) return DN_ENOSPC;
    {
        GemmGroup g;
        g.nprob = L;
        for (int m = 1; m <= L; ++m) {
            GemmProblem& p = g.p[m - 1];
            p = mk_problem(m == L ? c->fptr(c->o_Q[L]) : c->fptr(c->o_T[m]), c->ld[m], c->fptr(c->o_ZS[m - 1]),
                           c->ld[m - 1], c->fptr(c->o_tn) + pl.offset[m], c->ldw[m], c->dims[m], c->dims[m - 1] + 1, s);
            p.b_ones_col = 1;
            p.split_stride = (long long)c->dims[m] * c->ldw[m];
        }
        ProfScope ps(c, KC_GEMM_TN_MATVEC);
        DN_HIP(c, ps.err);
        DN_HIP(c, (launch_gemm<RT, RT, KC_GEMM_TN_MATVEC>(g, pl.tile, pl.splits, c->stream)));
        DN_HIP(c, ps.end());
    }
    return tn_reduce(c, &pl, false, v, out, 2.0 / (double)s);
}

int dn_profile_enable(dn_ctx* c, int on) {
    if (!c) return DN_EINVAL;
    if (!on && c->prof) DN_HIP(c, prof_fold(c));
    c->prof = on != 0;
    return DN_OK;
}

int dn_profile_select(dn_ctx* c, unsigned long long class_mask) {
    if (!c) return DN_EINVAL;
    DN_HIP(c, prof_fold(c));
    c->prof_mask = class_mask;
    return DN_OK;
}

int dn_profile_reset(dn_ctx* c) {
    if (!c) return DN_EINVAL;
    DN_HIP(c, prof_fold(c));
    for (int k = 0; k < KC_COUNT; ++k) {
        c->prof_ms[k] = 0.0;
        c->prof_n[k] = 0;
    }
    return DN_OK;
}

int dn_profile_num_classes(void) { return KC_COUNT; }

const char* dn_profile_class_name(int which) {
    return (which >= 0 && which < KC_COUNT) ? kClassNames[which] : nullptr;
}

int dn_profile_read(dn_ctx* c, int which, double* total_ms_host, long long* launches_host) {
    if (!c || which < 0 || which >= KC_COUNT || !total_ms_host || !launches_host) return DN_EINVAL;
    DN_HIP(c, prof_fold(c));
    *total_ms_host = c->prof_ms[which];
    *launches_host = c->prof_n[which];
    return DN_OK;
}

}  // extern "C"
