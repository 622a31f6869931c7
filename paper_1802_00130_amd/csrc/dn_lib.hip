// libdn: host side of the C-ABI declared in include/dn.h.  Validates arguments, lays out the
// caller's workspace, and enqueues the HIP kernels of dn_gemm.h / dn_kernels.h on one stream.
#include "dn_host_ctx.h"
#include "dn_host_gemm.h"
#include "dn_host_workspace.h"
#include "dn_host_product.h"
#include "dn_host_cg.h"


// Scratch of dn_forward_static: device memory that exists without any allocation call.  One copy per GPU, at an
// address of its own on each; host code never uses the array's name as an address, only what hipGetSymbolAddress
// returned for the device that is current.
static __device__ __align__(256) unsigned char scratch[DN_STATIC_SCRATCH_BYTES];

namespace {

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices] = {nullptr};

// device address of `scratch` on the current device (looked up once per device)
hipError_t static_scratch(void** out) {
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* ptr = nullptr;
        e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!ptr) return hipErrorInvalidSymbol;
        g_scratch_ptr[dev] = ptr;
    }
    *out = g_scratch_ptr[dev];
    return hipSuccess;
}

bool valid_network(int L, const int* dims, double C) {
    if (!dims || L < 1 || L > DN_MAX_LAYERS || !(C > 0.0)) return false;
    for (int m = 0; m <= L; ++m)
        if (dims[m] < 1) return false;
    return true;
}

// sizes, strides and theta offsets of the network (Section 2.1); no workspace map yet
void init_network(dn_ctx* c, int L, const int* dims, double C, int l_max, int s_max) {
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
}

}  // namespace

// ================================================================================================
extern "C" {

const char* dn_strerror(int code) {
    switch (code) {
        case DN_OK: return "ok";
        case DN_EINVAL: return "invalid argument";
        case DN_ENOSPC: return "workspace too small";
        case DN_ETOOBIG: return "problem exceeds the fixed scratch of the call that allocates nothing";
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
    if (!valid_network(L, dims, C) || l_max < 1 || s_max < 1) return DN_EINVAL;
    // row counts of the batched sweeps are int: s_max * n_L rows
    if ((long long)s_max * dims[L] > 0x7fffffffLL) return DN_EINVAL;
    dn_ctx* c = new (std::nothrow) dn_ctx();
    if (!c) return DN_ENOMEM;
    init_network(c, L, dims, C, l_max, s_max);
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

int dn_product_slices(const dn_ctx* c, int s) {
    if (!c || s < 1 || s > c->s_max) return DN_EINVAL;
    const TnPlan pl = plan_tn_product(c, s);
    return pl.total <= c->tn_floats ? pl.splits : DN_ENOSPC;
}

int dn_gemm_large_tiles(int nprob, const int* M, const int* N, const int* K, int* large) {
    if (!M || !N || !K || !large || nprob < 1 || nprob > DN_MAX_GROUP) return DN_EINVAL;
    GemmGroup g;
    g.nprob = nprob;
    for (int i = 0; i < nprob; ++i) {
        if (M[i] < 1 || N[i] < 1 || K[i] < 1) return DN_EINVAL;
        g.p[i] = mk_problem(nullptr, K[i], nullptr, K[i], nullptr, N[i], M[i], N[i], K[i]);
    }
    const unsigned mask = pick_128(g);
    int count = 0;
    for (int i = 0; i < nprob; ++i) {
        large[i] = (mask >> i) & 1u;
        count += large[i];
    }
    return count;
}

int dn_bind(dn_ctx* c, void* d_workspace, size_t bytes, void* hip_stream) {
    if (!c || !d_workspace) return DN_EINVAL;
    if ((reinterpret_cast<uintptr_t>(d_workspace) & 255u) != 0) return DN_EINVAL;
    if (bytes < c->ws_bytes) return DN_ENOSPC;
    c->ws = static_cast<char*>(d_workspace);
    c->stream = static_cast<hipStream_t>(hip_stream);
    c->bound = true;
    c->prepped = false;
    c->band_clean = false;
    c->fwd_valid = false;
    c->band_used = false;
    c->band_off = false;
    c->timeout_unreported = false;
    c->band_last_grid = 0;
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
    c->fwd_valid = false;
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

int dn_forward_static(int L, const int* dims, double C, const float* theta, const float* X, const float* Y, int l,
                      void* hip_stream, double* f_host, float* ZL) {
    if (!valid_network(L, dims, C) || !theta || !X || !Y || !f_host || l < 1) return DN_EINVAL;
    // a context on the stack (its containers stay empty: no profiling here), mapped onto the static scratch:
    // activations of the l rows, the two partial-sum arrays and the result word -- what dn_forward uses of a workspace
    dn_ctx ctx;
    dn_ctx* c = &ctx;
    init_network(c, L, dims, C, l, 1);
    size_t cur = 0;
    for (int m = 1; m <= L; ++m) {
        const unsigned long long bytes = sizeof(float) * (unsigned long long)l * (unsigned long long)c->ld[m];
        if (bytes > DN_STATIC_SCRATCH_BYTES) return DN_ETOOBIG;
        c->o_Zall[m] = take(cur, (size_t)bytes);
        if (cur > DN_STATIC_SCRATCH_BYTES) return DN_ETOOBIG;
    }
    for (int k = 0; k < 2; ++k) c->o_part[k] = take(cur, sizeof(double) * DN_MAX_PARTIALS);
    c->o_f = take(cur, 256);
    if (cur > DN_STATIC_SCRATCH_BYTES) return DN_ETOOBIG;
    c->ws_bytes = cur;
    void* base = nullptr;
    DN_HIP(c, static_scratch(&base));
    c->ws = static_cast<char*>(base);
    c->stream = static_cast<hipStream_t>(hip_stream);
    c->bound = true;
    int rc = forward_layers(c, theta, X, dims[0], l, c->o_Zall, L);
    if (rc != DN_OK) return rc;
    // every partial sum this call reads is written by it first (first chunk = overwrite), nothing has to start at zero
    return objective(c, theta, Y, l, l, true, true, nullptr, 0, ZL, f_host);
}

}  // extern "C"

namespace {

// Gradient (Section 2.2).  have_forward: the activations of these l <= l_max rows at this theta are already in
// the workspace (left there by the line search of the previous Newton step).
int grad_impl(dn_ctx* c, const float* theta, const float* X, const float* Y, int l, float* g, double* f_host,
              bool have_forward) {
    const int L = c->L, n0 = c->dims[0], nL = c->dims[L];
    if (L >= 2) {
        c->wt_of_prep = false;
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
            plans[m].floats[m] = tn_slice_floats(c, m);
            plans[m].offset[m] = tn_off;
            tn_off += round_up(plans[m].floats[m], 64);
        }
        if (tn_off > c->tn_floats) return DN_ENOSPC;
    }
    for (int r0 = 0; r0 < l; r0 += c->l_max) {
        const int rows = std::min(c->l_max, l - r0);
        const float* Xc = X + (long long)r0 * n0;
        int rc = have_forward ? DN_OK : forward_layers(c, theta, Xc, n0, rows, c->o_Zall, L);
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
                p.split_stride = tn_slice_floats(c, m);
                p.c_rows_padded = 1;
                p.accumulate = r0 > 0 ? 1 : 0;
                ProfScope ps(c, KC_GEMM_TN_GRAD);
                DN_HIP(c, ps.err);
                DN_HIP(c, (launch_gemm<RT, RT, KC_GEMM_TN_GRAD>(g1, plans[m].splits, c->stream)));
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
                ProfScope ps(c, KC_GEMM_BACK);
                DN_HIP(c, ps.err);
                DN_HIP(c, (launch_gemm<KC, KC, KC_GEMM_BACK>(g2, 1, c->stream)));
                DN_HIP(c, ps.end());
                cur ^= 1;
            }
        }
    }
    return tn_reduce(c, plans, true, theta, g, 1.0 / (double)l);
}

}  // namespace

extern "C" {

int dn_grad(dn_ctx* c, const float* theta, const float* X, const float* Y, int l, float* g, double* f_host) {
    if (!c || !theta || !X || !Y || !g || l < 1) return DN_EINVAL;
    if (!c->bound) return DN_ESTATE;
    c->fwd_valid = false;
    return grad_impl(c, theta, X, Y, l, g, f_host, false);
}

int dn_jacobian_prep(dn_ctx* c, const float* theta, const float* X, int l, const int* S, int s) {
    if (!c || !theta || !X || !S || l < 1 || s < 1 || s > c->s_max) return DN_EINVAL;
    if (!c->bound) return DN_ESTATE;
    const int L = c->L, nL = c->dims[L];
    c->prepped = false;
    {
        ProfScope ps(c, KC_GATHER);
        DN_HIP(c, ps.err);
        hipLaunchKernelGGL(gather_rows_kernel, dim3(std::min(cdiv(s, 4), 256 * 16)), dim3(256), 0, c->stream, X,
                           S, c->fptr(c->o_ZS[0]), s, c->dims[0], l, (long long)c->dims[0], c->ld[0]);
        DN_HIP(c, hipGetLastError());
        DN_HIP(c, ps.end());
    }
    // z^{m,i} for the hidden layers (the output layer's activations are not needed by the products)
    int rc = forward_layers(c, theta, c->fptr(c->o_ZS[0]), c->ld[0], s, c->o_ZS, L - 1);
    if (rc != DN_OK) return rc;
    {
        // [Z^m_S, 1]^T for the sums over samples of every later product (their right operand, K-contiguous)
        ProfScope ps(c, KC_GATHER);
        DN_HIP(c, ps.err);
        for (int m = 0; m < L; ++m) {
            hipLaunchKernelGGL(transpose_ones_kernel, dim3(cdiv(c->dims[m], 32), cdiv(s, 32)), dim3(256), 0, c->stream,
                               c->fptr(c->o_ZS[m]), c->ld[m], c->fptr(c->o_ZST[m]), c->ld_s, s, c->dims[m]);
            DN_HIP(c, hipGetLastError());
        }
        DN_HIP(c, ps.end());
    }
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
        c->wt_of_prep = false;
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
        ProfScope ps(c, KC_GEMM_PREP);
        DN_HIP(c, ps.err);
        DN_HIP(c, (launch_gemm<KC, KC, KC_GEMM_PREP>(g, 1, c->stream)));
        DN_HIP(c, ps.end());
    }
    c->s_cur = s;
    c->prepped = true;
    c->wt_of_prep = true;
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
    const bool have_forward = prm->reuse_forward && c->fwd_valid && c->fwd_theta == theta && c->fwd_X == X &&
                              c->fwd_Y == Y && c->fwd_l == l && l <= c->l_max;
    c->fwd_valid = false;
    int rc = grad_impl(c, theta, X, Y, l, g, &f0, have_forward);
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
        // the last objective evaluation was the accepted point: its activations are those of the new theta
        if (l <= c->l_max) {
            c->fwd_valid = true;
            c->fwd_theta = theta; c->fwd_X = X; c->fwd_Y = Y; c->fwd_l = l;
        }
    } else {
        st->alpha = 0.0;
        st->rho = 0.0;
        prm->lambda *= prm->boost;
    }
    st->f_new = f_new;
    DN_HIP(c, hipMemcpyAsync(d_prev, d, sizeof(float) * (size_t)n, hipMemcpyDeviceToDevice, c->stream));
    DN_HIP(c, hipStreamSynchronize(c->stream));
    return band_status(c);
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
    const int rc = band_status(c);
    if (rc != DN_OK) return rc;
    if (c->timeout_unreported) {
        c->timeout_unreported = false;
        return DN_ETIMEOUT;
    }
    return DN_OK;
}

int dn_gn_matvec_rop(dn_ctx* c, const float* v, float* out) {
    if (!c || !v || !out) return DN_EINVAL;
    if (!c->bound || !c->prepped) return DN_ESTATE;
    const int L = c->L, s = c->s_cur;
    const float* th = c->fptr(c->o_thS);
    // a gradient evaluated at another theta since dn_jacobian_prep has replaced the transposed weights
    if (L >= 2 && !c->wt_of_prep) {
        int rc = transpose_weights(c, th, 2, L);
        if (rc != DN_OK) return rc;
        c->wt_of_prep = true;
    }
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
        ProfScope ps(c, KC_GEMM_Q);
        DN_HIP(c, ps.err);
        DN_HIP(c, (launch_gemm<KC, KC, KC_GEMM_Q>(g, 1, c->stream)));
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
        ProfScope ps(c, KC_GEMM_ROP);
        DN_HIP(c, ps.err);
        DN_HIP(c, (launch_gemm<KC, KC, KC_GEMM_ROP>(g, 1, c->stream)));
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
        ProfScope ps(c, KC_GEMM_ROP);
        DN_HIP(c, ps.err);
        DN_HIP(c, (launch_gemm<KC, KC, KC_GEMM_ROP>(g, 1, c->stream)));
        DN_HIP(c, ps.end());
    }
    // 4. sums over samples for every layer, then out = v/C + (2/|S|) * sums
    TnPlan pl = plan_tn_product(c, s);
    if (pl.total > c->tn_floats) return DN_ENOSPC;
    {
        const float* left[DN_MAX_LAYERS + 1] = {nullptr};
        for (int m = 1; m <= L; ++m) left[m] = m == L ? c->fptr(c->o_Q[L]) : c->fptr(c->o_T[m]);
        const int rc = sums_over_samples(c, s, left, pl);
        if (rc != DN_OK) return rc;
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

int dn_profile_band_phases(dn_ctx* c, int on) {
    if (!c) return DN_EINVAL;
    c->band_clocks = on != 0;
    if (!on) c->band_last_grid = 0;
    return DN_OK;
}

int dn_profile_band_read(dn_ctx* c, double* cycles_host, double* bands_host) {
    if (!c || !cycles_host || !bands_host) return DN_EINVAL;
    if (!c->bound) return DN_ESTATE;
    cycles_host[0] = cycles_host[1] = cycles_host[2] = 0.0;
    *bands_host = 0.0;
    if (c->band_last_grid <= 0) return DN_OK;
    std::vector<unsigned long long> h;
    try {
        h.resize((size_t)c->band_last_grid * 4);
    } catch (const std::bad_alloc&) {
        return DN_ENOMEM;
    }
    DN_HIP(c, hipMemcpyAsync(h.data(), c->ws + c->o_bclk, sizeof(unsigned long long) * h.size(), hipMemcpyDeviceToHost,
                             c->stream));
    DN_HIP(c, hipStreamSynchronize(c->stream));
    double sum[3] = {0.0, 0.0, 0.0}, bands = 0.0;
    for (int b = 0; b < c->band_last_grid; ++b) {
        for (int k = 0; k < 3; ++k) sum[k] += (double)h[(size_t)b * 4 + k];
        bands += (double)h[(size_t)b * 4 + 3];
    }
    if (bands > 0.0)
        for (int k = 0; k < 3; ++k) cycles_host[k] = sum[k] / bands;
    *bands_host = bands / (double)c->band_last_grid;
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
