// Forward pass, objective, and the Gauss-Newton products (all block modes) as sequences of launches.
// Part of the one translation unit dn_lib.hip (helpers live in its unnamed namespace).
#pragma once
#include "dn_host_workspace.h"

namespace {

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
        ProfScope ps(c, KC_GEMM_FWD);
        DN_HIP(c, ps.err);
        g.p[0].sigmoid = m < c->L ? 1 : 0;
        DN_HIP(c, (launch_gemm<KC, KC, KC_GEMM_FWD>(g, 1, c->stream)));
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

// Work-groups of tn_reduce_kernel: layer m's items (row, 1024 columns) are shared by blk[m+1] - blk[m]
// work-groups, about 1000 in all (at most DN_MAX_PARTIALS: each may emit one partial sum).
int reduce_grid(const dn_ctx* c, int* blk /* L + 2 entries, index 1..L+1 */) {
    long long total = 0;
    for (int m = 1; m <= c->L; ++m) total += (long long)c->dims[m] * cdiv(c->dims[m - 1] + 1, 1024);
    int blocks = 0;
    for (int m = 1; m <= c->L; ++m) {
        const long long items = (long long)c->dims[m] * cdiv(c->dims[m - 1] + 1, 1024);
        blk[m] = blocks;
        blocks += (int)std::max<long long>(1, std::min<long long>(items, items * 1000 / total));
    }
    blk[c->L + 1] = blocks;
    return blocks;
}

// out = x/C + scale * (folded partial sums), theta layout.  dot (nullable): see tn_reduce_kernel.
int tn_reduce(dn_ctx* c, const TnPlan* plans /* indexed by layer, or one plan for all */, bool per_layer,
              const float* x, float* out, double scale, double* dot = nullptr, float lambda = 0.f) {
    ReduceArgs ra;
    std::memset(&ra, 0, sizeof(ra));
    ra.L = c->L;
    for (int m = 0; m <= c->L; ++m) ra.n[m] = c->dims[m];
    const int blocks = reduce_grid(c, ra.blk_begin);
    for (int m = 1; m <= c->L; ++m) {
        const TnPlan& pl = per_layer ? plans[m] : plans[0];
        ra.off[m] = c->woff[m];
        ra.W[m] = c->fptr(c->o_tn) + pl.offset[m];
        ra.ldw[m] = c->ldw[m];
        ra.split_stride[m] = tn_slice_floats(c, m);
        ra.splits[m] = pl.splits;
        ra.chunks[m] = cdiv(c->dims[m - 1] + 1, 1024);
        ra.items[m] = c->dims[m] * ra.chunks[m];
    }
    ProfScope ps(c, KC_TN_REDUCE);
    DN_HIP(c, ps.err);
    hipLaunchKernelGGL(tn_reduce_kernel, dim3(blocks), dim3(256), 0, c->stream, ra, x, out, (float)(1.0 / c->C),
                       (float)scale, dot, lambda);
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

// ---- single pass over the stored blocks by teams of work-groups: plumbing of jv_jtv_band_kernel ---------
// grid of the two-pass kernels when they are enqueued as the fall-back of the band kernel: they walk over their
// virtual work-groups, and a launch that finds nothing to do should cost next to nothing
constexpr int kFallbackGrid = 2048;

struct BandPlan {
    bool ok = false;
    int H = 0, GA = 1;
    BandArgs ba;
};

// resident work-groups per CU of kernel variant v (0: H = 16, 1: H = 28, 2: H = 16 with input groups)
hipError_t band_occupancy(dn_ctx* c, int v, int* wgs) {
    if (c->band_wgs_per_cu[v] == 0) {
        int nb = 0;
        hipError_t e = v == 0   ? hipOccupancyMaxActiveBlocksPerMultiprocessor(&nb, jv_jtv_band_kernel<16, 1, 4>, 256, 0)
                       : v == 1 ? hipOccupancyMaxActiveBlocksPerMultiprocessor(&nb, jv_jtv_band_kernel<28, 1, 3>, 256, 0)
                                : hipOccupancyMaxActiveBlocksPerMultiprocessor(&nb, jv_jtv_band_kernel<16, DN_MAX_SPLIT, 3>, 256, 0);
        if (e != hipSuccess) return e;
        c->band_wgs_per_cu[v] = nb >= 1 ? nb : -1;
    }
    *wgs = c->band_wgs_per_cu[v];
    return hipSuccess;
}

// Layers 1..L-2 (block L-1 is applied as dense products around the kernel).
// Q, T: per layer, the product's temporaries (partition mode: those of the input groups, one after another)
hipError_t plan_band(dn_ctx* c, int mode, const float* const* Q, float* const* T, BandPlan& bp) {
    bp.ok = false;
    const int L = c->L, nL = c->dims[L], s = c->s_cur;
    if (c->stream_passes == 2 || c->band_off) return hipSuccess;
    const int m_hi = L - 2;      // block L-1 is applied as dense products around the kernel in every mode
    if (m_hi < 1) return hipSuccess;
    BandArgs& ba = bp.ba;
    std::memset(&ba, 0, sizeof(ba));
    ba.L = L; ba.s = s; ba.nL = nL; ba.mode = mode;
    int ncs = 0;
    bool fits = true;
    auto add = [&](int m, int j0, int lo, int hi) {
        if (ncs < DN_MAX_BAND_SLICES) ba.sl[ncs] = BandSlice{m, j0, lo, hi, 0, 0};
        else fits = false;
        ++ncs;
    };
    for (int m = 1; m <= m_hi; ++m) {
        ba.ld[m] = c->ld[m];
        ba.P[m] = c->fptr(c->o_P[m]);
        ba.Q[m] = Q[m];
        ba.T[m] = T[m];
        ba.ga[m] = mode == DN_PARTITION ? c->split[m - 1] : 1;
        // column slices never straddle an output group (partition mode; otherwise the layer is one group); the slices of
        // a group share their sums (per-layer and partition mode; the whole matrix: all slices, set below)
        const int groups = mode == DN_PARTITION ? c->split[m] : 1;
        for (int y = 0; y < groups; ++y) {
            const int glo = mode == DN_PARTITION ? c->gbound[m][y] : 0;
            const int ghi = mode == DN_PARTITION ? c->gbound[m][y + 1] : c->dims[m];
            const int first = ncs;
            for (int j0 = glo & ~3; j0 < ghi; j0 += 1024) add(m, j0, std::max(glo, j0), std::min(ghi, j0 + 1024));
            for (int k = first; k < std::min(ncs, DN_MAX_BAND_SLICES); ++k) { ba.sl[k].c_lo = first; ba.sl[k].c_hi = ncs; }
        }
    }
    if (!fits) return hipSuccess;
    if (mode == DN_FULL)
        for (int k = 0; k < ncs; ++k) { ba.sl[k].c_lo = 0; ba.sl[k].c_hi = ncs; }
    ba.ld[L] = c->ld[L];
    ba.Q[L] = Q[L];
    ba.T[L] = T[L];
    ba.ga[L] = mode == DN_PARTITION ? c->split[L - 1] : 1;
    // rows per band: as equal as possible, at most 28 (16 with input groups: more vectors per thread)
    const int hmax = mode == DN_PARTITION ? 16 : 28;
    ba.nrs = cdiv(nL, hmax);
    ba.rps = cdiv(nL, ba.nrs);
    bp.GA = mode == DN_PARTITION ? DN_MAX_SPLIT : 1;
    bp.H = ba.rps <= 16 ? 16 : 28;
    int wgs = 0;
    hipError_t e = band_occupancy(c, mode == DN_PARTITION ? 2 : (bp.H == 16 ? 0 : 1), &wgs);
    if (e != hipSuccess) return e;
    if (wgs < 1) return hipSuccess;
    const int resident = std::min(kMaxResidentWGs, c->num_cus * wgs);
    const int teams_max = std::min(s, resident / ncs);
    if (teams_max < 1) return hipSuccess;
    // as many teams as fit (measured: fewer teams with an even share of the samples each are no faster)
    ba.ncs = ncs;
    ba.teams = teams_max;
    ba.part = reinterpret_cast<unsigned long long*>(c->ws + c->o_texch);
    ba.error = reinterpret_cast<unsigned*>(c->ws + c->o_terr);
    ba.spin_limit = c->spin_limit;
    ba.clk = c->band_clocks ? reinterpret_cast<unsigned long long*>(c->ws + c->o_bclk) : nullptr;
    bp.ok = true;
    return hipSuccess;
}

hipError_t launch_band(dn_ctx* c, BandPlan& bp) {
    BandArgs& ba = bp.ba;
    ba.per_launch = (unsigned)cdiv(ba.s, ba.teams) * (unsigned)ba.nrs + 1u;
    ba.exch_words = kBandExchWords;
    ba.seq = reinterpret_cast<unsigned*>(c->ws + c->o_terr) + 16;
    if (!c->band_clean) {
        // first use after dn_bind: exchange words, error word and sequence base start from a blank slate
        hipLaunchKernelGGL(band_clear_kernel, dim3(1024), dim3(256), 0, c->stream, ba.part, kBandExchWords, ba.error,
                           ba.seq);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
        c->band_clean = true;
    }
    c->band_used = true;
    const dim3 grid(ba.teams * ba.ncs), block(256);
    if (ba.clk) c->band_last_grid = (int)grid.x;
    if (ba.clk) {
        // the variants with phase clocks (a diagnostic: they need a few registers more)
        if (bp.GA > 1)       hipLaunchKernelGGL((jv_jtv_band_kernel<16, DN_MAX_SPLIT, 3, true>), grid, block, 0, c->stream, ba);
        else if (bp.H == 16) hipLaunchKernelGGL((jv_jtv_band_kernel<16, 1, 4, true>), grid, block, 0, c->stream, ba);
        else                 hipLaunchKernelGGL((jv_jtv_band_kernel<28, 1, 3, true>), grid, block, 0, c->stream, ba);
    } else if (bp.GA > 1)    hipLaunchKernelGGL((jv_jtv_band_kernel<16, DN_MAX_SPLIT, 3>), grid, block, 0, c->stream, ba);
    else if (bp.H == 16)     hipLaunchKernelGGL((jv_jtv_band_kernel<16, 1, 4>), grid, block, 0, c->stream, ba);
    else                     hipLaunchKernelGGL((jv_jtv_band_kernel<28, 1, 3>), grid, block, 0, c->stream, ba);
    return hipGetLastError();
}

// After a synchronisation: has a wait of the band kernel run out?  The products were completed by the two-pass
// kernels enqueued behind it; from now on (until dn_bind) the context uses those directly.
int band_status(dn_ctx* c) {
    if (!c->band_used || c->band_off) return DN_OK;
    unsigned err = 0;
    DN_HIP(c, hipMemcpyAsync(&err, c->ws + c->o_terr, sizeof(err), hipMemcpyDeviceToHost, c->stream));
    DN_HIP(c, hipStreamSynchronize(c->stream));
    if (err) {
        c->band_off = true;
        c->timeout_unreported = true;
    }
    return DN_OK;
}

int gn_matvec_part(dn_ctx* c, const float* v, float* out);

// Sums over samples of a product, all layers in one launch: W_m = left_m^T [Z^{m-1}, 1] into the partial-sum buffer
// (left_m = T^m: s rows of ld[m] floats).  The right operand was transposed once by dn_jacobian_prep (K-contiguous,
// the ones of the bias terms as a real row).  The left one is new in every product and normally goes through the
// transposing loads of the tile engine; when the launch is large enough for the 128 x 128 tiles, it is transposed
// first (one pass over s x sum n_m floats) and both operands are read K-contiguously: 4096 x 5 - 1000, 2000 samples,
// 2.57 -> 2.42 ms including the copy (49 us).
int sums_over_samples(dn_ctx* c, int s, const float* const* left, const TnPlan& pl) {
    const int L = c->L;
    GemmGroup g;
    g.nprob = L;
    if (pl.splits == 1) {
        for (int m = 1; m <= L; ++m) {
            GemmProblem& p = g.p[m - 1];
            p = mk_problem(c->fptr(c->o_TT[m]), c->ld_s, c->fptr(c->o_ZST[m - 1]), c->ld_s,
                           c->fptr(c->o_tn) + pl.offset[m], c->ldw[m], c->dims[m], c->dims[m - 1] + 1, s);
            p.split_stride = tn_slice_floats(c, m);
        }
        if (pick_128(g) != 0) {
            TransposeArgs ta;
            std::memset(&ta, 0, sizeof(ta));
            ta.nprob = L;
            ta.rows = s;
            ta.tiles_r = cdiv(s, 64);
            ta.ld_dst = c->ld_s;
            int blocks = 0;
            for (int m = 1; m <= L; ++m) {
                ta.src[m - 1] = left[m];
                ta.dst[m - 1] = c->fptr(c->o_TT[m]);
                ta.ld_src[m - 1] = c->ld[m];
                ta.cols[m - 1] = c->dims[m];
                ta.first[m - 1] = blocks;
                blocks += ta.tiles_r * cdiv(c->dims[m], 64);
            }
            ta.first[L] = blocks;
            ProfScope ps(c, KC_GEMM_TN_MATVEC);
            DN_HIP(c, ps.err);
            hipLaunchKernelGGL(transpose_group_kernel, dim3(blocks), dim3(256), 0, c->stream, ta);
            DN_HIP(c, hipGetLastError());
            DN_HIP(c, (launch_gemm<KC, KC, KC_GEMM_TN_MATVEC>(g, 1, c->stream)));
            DN_HIP(c, ps.end());
            return DN_OK;
        }
    }
    for (int m = 1; m <= L; ++m) {
        GemmProblem& p = g.p[m - 1];
        p = mk_problem(left[m], c->ld[m], c->fptr(c->o_ZST[m - 1]), c->ld_s, c->fptr(c->o_tn) + pl.offset[m],
                       c->ldw[m], c->dims[m], c->dims[m - 1] + 1, s);
        p.split_stride = tn_slice_floats(c, m);
        p.c_rows_padded = 1;
    }
    ProfScope ps(c, KC_GEMM_TN_MATVEC);
    DN_HIP(c, ps.err);
    DN_HIP(c, (launch_gemm<RT, KC, KC_GEMM_TN_MATVEC>(g, pl.splits, c->stream)));
    DN_HIP(c, ps.end());
    return DN_OK;
}

// out = G^S v (mode full / per-layer), Section 4.2 factored products on the stored blocks
// dot, lambda: passed on to the fold of the sums over samples (not in partition mode)
int gn_matvec(dn_ctx* c, const float* v, float* out, int mode, double* dot = nullptr, float lambda = 0.f) {
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
        // Small launches (a few tiles per CU) whose longest sum over t is at least twice any other: cut that
        // layer's sum in two halves, written to Q^m and a second buffer that the fused kernel adds on the way
        // in.  The launch then consists of tiles of similar length (measured at 784-300-300-10, |S| = 3000:
        // 30.2 -> 26.8 us; at 3072-1000-500-10, 1000 tiles, it gains nothing: 173 -> 176 us).
        if (fused && L < DN_MAX_GROUP && group_tiles(g, 64, 64) <= 3 * c->num_cus) {
            int big = 0;                       // among the hidden layers: Q^L is read as it is
            for (int k = 1; k + 1 < L; ++k)
                if (g.p[k].K > g.p[big].K) big = k;
            int other = 0;
            for (int k = 0; k < L; ++k)
                if (k != big) other = std::max(other, g.p[k].K);
            if (g.p[big].K >= 512 && g.p[big].K >= 2 * other) {
                const int kh = (int)round_up(g.p[big].K / 2, 16);
                // the second half right behind the first, so that the walk still has its longest tiles first
                for (int k = g.nprob; k > big + 1; --k) g.p[k] = g.p[k - 1];
                ++g.nprob;
                GemmProblem& second = g.p[big + 1];
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
        DN_HIP(c, (launch_gemm<KC, KC, KC_GEMM_Q>(g, 1, c->stream)));
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
            DN_HIP(c, (launch_gemm<KC, KC, KC_GEMM_IMPLICIT>(g, 1, c->stream)));
            DN_HIP(c, ps.end());
        }
        BandPlan bp;
        {
            const float* Qv[DN_MAX_LAYERS + 1] = {nullptr};
            float* Tv[DN_MAX_LAYERS + 1] = {nullptr};
            for (int m = 1; m <= L; ++m) { Qv[m] = c->fptr(c->o_Q[m]); Tv[m] = c->fptr(c->o_T[m]); }
            DN_HIP(c, plan_band(c, mode, Qv, Tv, bp));
        }
        int chunks = 1;
        for (int m = 1; m + 1 < L; ++m) chunks += cdiv(c->dims[m], 1024);
        constexpr int UB = 16;
        if (bp.ok) {
            // one read of the stored blocks: teams of work-groups, see jv_jtv_band_kernel; behind it the two-pass
            // kernels, which leave at once unless a wait of the band kernel ran out
            ProfScope ps(c, KC_JV_JTV_BAND);
            DN_HIP(c, ps.err);
            DN_HIP(c, launch_band(c, bp));
            hipLaunchKernelGGL(jv_rows_kernel<UB>, dim3(std::min(s * cdiv(nL, UB), kFallbackGrid)), dim3(256), 0, c->stream,
                               a, bp.ba.error);
            DN_HIP(c, hipGetLastError());
            hipLaunchKernelGGL(jtv_cols_kernel, dim3((unsigned)std::min<long long>((long long)s * chunks, kFallbackGrid)),
                               dim3(256), sizeof(float) * nL, c->stream, a, chunks, bp.ba.error);
            DN_HIP(c, hipGetLastError());
            DN_HIP(c, ps.end());
        } else {
            {
                ProfScope ps(c, KC_JV);
                DN_HIP(c, ps.err);
                hipLaunchKernelGGL(jv_rows_kernel<UB>, dim3(s * cdiv(nL, UB)), dim3(256), 0, c->stream, a,
                                   (const unsigned*)nullptr);
                DN_HIP(c, hipGetLastError());
                DN_HIP(c, ps.end());
            }
            {
                ProfScope ps(c, KC_JTV);
                DN_HIP(c, ps.err);
                hipLaunchKernelGGL(jtv_cols_kernel, dim3((unsigned)((long long)s * chunks)), dim3(256),
                                   sizeof(float) * nL, c->stream, a, chunks, (const unsigned*)nullptr);
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
            DN_HIP(c, (launch_gemm<KC, RT, KC_GEMM_IMPLICIT>(g, 1, c->stream)));
            DN_HIP(c, ps.end());
        }
    }
    // 3. sums over samples for every layer
    TnPlan pl = plan_tn_product(c, s);
    if (pl.total > c->tn_floats) return DN_ENOSPC;
    {
        const float* left[DN_MAX_LAYERS + 1] = {nullptr};
        for (int m = 1; m <= L; ++m) left[m] = c->fptr(c->o_T[m]);
        const int rc = sums_over_samples(c, s, left, pl);
        if (rc != DN_OK) return rc;
    }
    // 4. fold slices, scale by 1/|S|, add v/C
    return tn_reduce(c, &pl, false, v, out, 1.0 / (double)s, dot, lambda);
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
    // where the partial sums of p^T A p come from: the fold of the product (full and per-layer systems: its
    // work-groups are grouped by layer), or cg_dot_gather_kernel on this grid (partitions)
    if (mode == DN_PARTITION) {
        for (int k = 0; k <= sg.nseg; ++k) sg.pb[k] = sg.cb[k];
    } else {
        int blk[DN_MAX_LAYERS + 2];
        const int blocks = reduce_grid(c, blk);
        if (mode == DN_BLOCKDIAG) {
            for (int m = 1; m <= c->L + 1; ++m) sg.pb[m - 1] = blk[m];
        } else {
            sg.pb[0] = 0;
            sg.pb[1] = blocks;
        }
    }
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
    // 2. the passes over the stored blocks: one pass when a sample's strips fit one work-group's registers
    //    (as in the other modes), else the general two-pass kernels
    {
        // strip slots: up to 256 columns of one output group of one layer, from the multiple of four at or
        // below the group's first column
        int w = 0;
        for (int m = 1; m < L; ++m)
            for (int y = 0; y < c->split[m]; ++y)
                for (int col = c->gbound[m][y] & ~3; col < c->gbound[m][y + 1]; col += 256, ++w)
                    if (w < DN_MAX_WSLOTS) {
                        a.wlayer[w] = m;
                        a.wcol[w] = col;
                        a.wgrp[w] = y;
                    }
        a.nwslots = w;
    }
    const bool fused = L >= 2 && c->stream_passes != 2 &&
                       ((nL <= 16 && a.nwslots <= 16) || (nL <= 8 && a.nwslots <= DN_MAX_WSLOTS));
    // 1. inner sums over t, one product per (layer, input group); the bias term rides with group 0
    {
        GemmGroup g;
        g.nprob = 0;
        auto flush = [&]() -> int {
            if (g.nprob == 0) return DN_OK;
            ProfScope ps(c, KC_GEMM_Q);
            DN_HIP(c, ps.err);
            DN_HIP(c, (launch_gemm<KC, KC, KC_GEMM_Q>(g, 1, c->stream)));
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
                if (!fused && L >= 2 && m == L - 1) {
                    // outside the register-strip kernel block L-1 = A^L diag(sigma') is applied as dense products: its
                    // q leaves this product already scaled by sigma'(s^{L-1})
                    p.aux = c->fptr(c->o_ZS[L - 1]);
                    p.ldaux = c->ld[L - 1];
                }
                if (g.nprob == DN_MAX_GROUP) {
                    const int rc = flush();
                    if (rc != DN_OK) return rc;
                }
            }
        const int rc = flush();
        if (rc != DN_OK) return rc;
    }
    if (fused) {
        ProfScope ps(c, KC_JV_JTV_FUSED);
        DN_HIP(c, ps.err);
        const dim3 grid(s), block(64 * std::min(a.nwslots, 16));
        a.ga_max = a.gb_max = 1;
        for (int m = 1; m < L; ++m) {
            a.ga_max = std::max(a.ga_max, c->split[m - 1]);
            a.gb_max = std::max(a.gb_max, c->split[m]);
        }
        // LDS: partial sums per (strip slot, input group, output), then r per (layer, input group, output group, output)
        const int nlmax = a.nwslots <= 16 ? (nL <= 4 ? 4 : nL <= 8 ? 8 : nL <= 12 ? 12 : 16) : (nL <= 4 ? 4 : 8);
        const size_t lds = sizeof(float) * ((size_t)a.nwslots + (size_t)(L - 1) * a.gb_max) * a.ga_max * nlmax;
        if (a.nwslots <= 16) {
            if (nL <= 4)       hipLaunchKernelGGL((jv_jtv_fused_part_kernel<4, 1>), grid, block, lds, c->stream, a);
            else if (nL <= 8)  hipLaunchKernelGGL((jv_jtv_fused_part_kernel<8, 1>), grid, block, lds, c->stream, a);
            else if (nL <= 12) hipLaunchKernelGGL((jv_jtv_fused_part_kernel<12, 1>), grid, block, lds, c->stream, a);
            else               hipLaunchKernelGGL((jv_jtv_fused_part_kernel<16, 1>), grid, block, lds, c->stream, a);
        } else {
            if (nL <= 4)       hipLaunchKernelGGL((jv_jtv_fused_part_kernel<4, 2>), grid, block, lds, c->stream, a);
            else               hipLaunchKernelGGL((jv_jtv_fused_part_kernel<8, 2>), grid, block, lds, c->stream, a);
        }
        DN_HIP(c, hipGetLastError());
        DN_HIP(c, ps.end());
    } else {
        // Block L-1 = A^L diag(sigma') is not streamed: per partition (a, b) of layer L-1 two small dense products
        // with the columns T_b of A^L stand in for it (q^{L-1,a} came out of step 1 scaled by sigma'):
        //   before the passes  r^{(a,b)} = (sigma' q^{L-1,a})[:, T_b] A^L[:, T_b]^T,
        //   after them         t^{L-1,a}[:, T_b] = sigma' * (2 r^{(a,b)} A^L[:, T_b]).
        const long long slab = (long long)s * c->ldr;
        auto implicit_block = [&](bool before) -> int {
            if (L < 2) return DN_OK;
            const int ga = c->split[L - 2], gb = c->split[L - 1];
            GemmGroup g;
            g.nprob = 0;
            auto flush = [&]() -> int {
                if (g.nprob == 0) return DN_OK;
                ProfScope ps(c, KC_GEMM_IMPLICIT);
                DN_HIP(c, ps.err);
                if (before) DN_HIP(c, (launch_gemm<KC, KC, KC_GEMM_IMPLICIT>(g, 1, c->stream)));
                else        DN_HIP(c, (launch_gemm<KC, RT, KC_GEMM_IMPLICIT>(g, 1, c->stream)));
                DN_HIP(c, ps.end());
                g.nprob = 0;
                return DN_OK;
            };
            for (int x = 0; x < ga; ++x)
                for (int y = 0; y < gb; ++y) {
                    const int t0 = c->gbound[L - 1][y], t1 = c->gbound[L - 1][y + 1];
                    float* r = c->fptr(c->o_Rp) + (long long)(c->part_base[L - 1] + x * gb + y) * slab;
                    GemmProblem& p = g.p[g.nprob++];
                    if (before) {
                        p = mk_problem(c->fptr(c->o_Qp[L - 1]) + (long long)x * s * c->ld[L - 1] + t0, c->ld[L - 1],
                                       c->fptr(c->o_AL) + t0, c->ld[L - 1], r, c->ldr, s, nL, t1 - t0);
                    } else {
                        p = mk_problem(r, c->ldr, c->fptr(c->o_AL) + t0, c->ld[L - 1],
                                       c->fptr(c->o_Tp[L - 1]) + (long long)x * s * c->ld[L - 1] + t0, c->ld[L - 1], s, t1 - t0,
                                       nL);
                        p.aux = c->fptr(c->o_ZS[L - 1]) + t0;
                        p.ldaux = c->ld[L - 1];
                        p.alpha = 2.0f;
                    }
                    if (g.nprob == DN_MAX_GROUP) {
                        const int rc = flush();
                        if (rc != DN_OK) return rc;
                    }
                }
            return flush();
        };
        int rc = implicit_block(true);
        if (rc != DN_OK) return rc;
        a.m_hi = L - 2;
        int chunks = 1;
        for (int m = 1; m <= a.m_hi; ++m) chunks += cdiv(c->dims[m], 1024);
        int most = 1;
        for (int m = 1; m <= a.m_hi; ++m) most = std::max(most, c->split[m - 1] * c->split[m]);
        const size_t lds = sizeof(float) * (size_t)most * nL;
        BandPlan bp;
        {
            const float* Qv[DN_MAX_LAYERS + 1] = {nullptr};
            float* Tv[DN_MAX_LAYERS + 1] = {nullptr};
            for (int m = 1; m <= L; ++m) { Qv[m] = c->fptr(c->o_Qp[m]); Tv[m] = c->fptr(c->o_Tp[m]); }
            DN_HIP(c, plan_band(c, DN_PARTITION, Qv, Tv, bp));
        }
        if (bp.ok) {
            // one read of the stored blocks (teams of work-groups), the two-pass kernels behind it as the fall-back
            ProfScope ps(c, KC_JV_JTV_BAND);
            DN_HIP(c, ps.err);
            DN_HIP(c, launch_band(c, bp));
            hipLaunchKernelGGL((jv_part_kernel<2>), dim3(std::min(s * cdiv(nL, 8), kFallbackGrid)), dim3(256), 0, c->stream,
                               a, bp.ba.error);
            DN_HIP(c, hipGetLastError());
            hipLaunchKernelGGL(jtv_part_kernel, dim3((unsigned)std::min<long long>((long long)s * chunks, kFallbackGrid)),
                               dim3(256), lds, c->stream, a, chunks, bp.ba.error);
            DN_HIP(c, hipGetLastError());
            DN_HIP(c, ps.end());
        } else {
            if (a.m_hi >= 1) {
                ProfScope ps(c, KC_JV);
                DN_HIP(c, ps.err);
                hipLaunchKernelGGL((jv_part_kernel<2>), dim3(s * cdiv(nL, 8)), dim3(256), 0, c->stream, a,
                                   (const unsigned*)nullptr);
                DN_HIP(c, hipGetLastError());
                DN_HIP(c, ps.end());
            }
            ProfScope ps(c, KC_JTV);
            DN_HIP(c, ps.err);
            hipLaunchKernelGGL(jtv_part_kernel, dim3((unsigned)((long long)s * chunks)), dim3(256), lds, c->stream, a,
                               chunks, (const unsigned*)nullptr);
            DN_HIP(c, hipGetLastError());
            DN_HIP(c, ps.end());
        }
        rc = implicit_block(false);
        if (rc != DN_OK) return rc;
    }
    // 3. sums over samples, one product per (layer, input group) into that group's columns; bias sums apart
    TnPlan pl = plan_tn_product(c, s);
    if (pl.total > c->tn_floats) return DN_ENOSPC;
    {
        GemmGroup g;
        g.nprob = 0;
        auto flush = [&]() -> int {
            if (g.nprob == 0) return DN_OK;
            ProfScope ps(c, KC_GEMM_TN_MATVEC);
            DN_HIP(c, ps.err);
            DN_HIP(c, (launch_gemm<RT, KC, KC_GEMM_TN_MATVEC>(g, pl.splits, c->stream)));
            DN_HIP(c, ps.end());
            g.nprob = 0;
            return DN_OK;
        };
        for (int m = 1; m <= L; ++m)
            for (int x = 0; x < c->split[m - 1]; ++x) {
                const int t0 = c->gbound[m - 1][x], t1 = c->gbound[m - 1][x + 1];
                GemmProblem& p = g.p[g.nprob++];
                p = mk_problem(c->fptr(c->o_Tp[m]) + (long long)x * s * c->ld[m], c->ld[m],
                               c->fptr(c->o_ZST[m - 1]) + (long long)t0 * c->ld_s, c->ld_s,
                               c->fptr(c->o_tn) + pl.offset[m] + t0, c->ldw[m], c->dims[m], t1 - t0, s);
                p.split_stride = tn_slice_floats(c, m);
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
            ba.slice[m] = tn_slice_floats(c, m);
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
