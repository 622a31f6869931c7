// Context of the library: limits, kernel classes for the profile, the workspace map, error and profile helpers.
// Part of the one translation unit dn_lib.hip (helpers live in its unnamed namespace).
#pragma once

#include "../../include/dn.h"

#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstdint>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <new>
#include <vector>

#include "dn_gemm.h"
#include "dn_kernels.h"

using namespace dn;

namespace {

// K-tile depths; slices of split sums are cut at multiples of the deepest
constexpr int kBKmax = 32;
// tile rows per super-row of the tile walk: 8 x 8 tiles are about what one XCD (32 CUs) holds at a time
constexpr int kGroupM = 8;
// most work-groups of 256 threads a launch can have resident on the chip (256 CUs x 2048 threads / 256);
// sizes the exchange buffer of the band kernel
constexpr int kMaxResidentWGs = 2048;
// 64-bit words of the band kernel's exchange buffer: 2 sets x (teams x slices <= kMaxResidentWGs work-groups) x
// (at most DN_MAX_SPLIT input groups) x (32 rows per band)
constexpr long long kBandExchWords = 2LL * kMaxResidentWGs * DN_MAX_SPLIT * 32;

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
    KC_JV_JTV_BAND,       // product: both passes over P, one read, teams of work-groups (plus their idle fall-back)
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
    "jv_jtv_fused", "jv_rows", "jtv_cols", "jv_jtv_band", "gemm_implicit_block", "gemm_rop_sweeps", "tn_reduce", "jac_init", "gather_rows", "loss", "cg_vector"};

inline long long round_up(long long x, long long a) { return (x + a - 1) / a * a; }
inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
inline int cdiv(long long a, long long b) { return (int)((a + b - 1) / b); }

struct TnPlan {
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
    size_t o_ZST[DN_MAX_LAYERS + 1] = {0};   // [Z^m_S, 1]^T: (n_m + 1) rows of ld_s floats, m = 0..L-1
    long long ld_s = 0;                      // row stride of those: s_max rounded up to 4
    size_t o_TT[DN_MAX_LAYERS + 1] = {0};    // (T^m)^T: n_m rows of ld_s floats, m = 1..L (large products only)
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
    // band kernel: exchange words, error word
    size_t o_texch = 0, o_terr = 0, o_bclk = 0;
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
    long long tn_floats = 0;

    char* ws = nullptr;
    hipStream_t stream = nullptr;
    bool bound = false;
    bool prepped = false;
    int s_cur = 0;
    int last_hip = 0;
    int num_cus = 256;
    // band kernel (single pass over the stored blocks where the register-strip kernel does not fit)
    int stream_passes = 0;          // 0 automatic, 2 force the two-pass kernels
    unsigned spin_limit = 1u << 20;
    bool band_clean = false;        // exchange words and error word cleared since the last dn_bind
    bool band_used = false;
    bool band_off = false;          // a wait ran out since the last dn_bind: two-pass kernels from now on
    bool timeout_unreported = false;   // ... and dn_sync_status has not said so yet
    bool band_clocks = false;       // collect the phase clocks of the band kernel (dn_profile_band_phases)
    int band_last_grid = 0;         // work-groups of the last band launch made with the clocks on
    int band_wgs_per_cu[3] = {0, 0, 0};   // resident work-groups per CU of each kernel variant (0: not looked up)

    // profiling
    bool prof = false;
    unsigned long long prof_mask = ~0ull;
    double prof_ms[KC_COUNT] = {0};
    long long prof_n[KC_COUNT] = {0};
    struct Pending { int cls; hipEvent_t a, b; };
    std::vector<Pending> pending;
    std::vector<hipEvent_t> free_events;

    // activations of all l rows left in the workspace by the last accepted line-search point of dn_newton_step
    bool fwd_valid = false;
    const float* fwd_theta = nullptr;
    const float* fwd_X = nullptr;
    const float* fwd_Y = nullptr;
    int fwd_l = 0;

    // the transposed weights in the workspace are those of the theta saved by the last dn_jacobian_prep
    // (a gradient at another theta overwrites them; the R-operator product restores them before use)
    bool wt_of_prep = false;

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

}  // namespace
