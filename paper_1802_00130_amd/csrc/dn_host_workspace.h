// Map of the caller's workspace and small launch helpers.
// Part of the one translation unit dn_lib.hip (helpers live in its unnamed namespace).
#pragma once
#include "dn_host_gemm.h"

namespace {

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
    c->ld_s = round_up(c->s_max, 4);
    for (int m = 0; m < L; ++m) c->o_ZST[m] = take(cur, sizeof(float) * (size_t)(c->dims[m] + 1) * c->ld_s);
    for (int m = 1; m <= L; ++m) c->o_TT[m] = take(cur, sizeof(float) * (size_t)c->dims[m] * c->ld_s);
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
    // partial sums over samples: the product's slice count is not monotone in the number of samples, so take the
    // largest plan of any s <= s_max (scanned with a stride for very large s_max; plan_tn_product cuts a plan
    // back if a count in between asks for more)
    long long tn = plan_tn(c, c->s_max, true, 0).total;
    for (int s = 1, stride = std::max(1, c->s_max / 16384); s < c->s_max; s += stride)
        tn = std::max(tn, plan_tn(c, s, true, 0).total);
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
    // band kernel: exchange words (sequence number + value)
    if (L >= 3) c->o_texch = take(cur, sizeof(unsigned long long) * kBandExchWords);
    c->o_terr = take(cur, 256);
    c->o_bclk = take(cur, sizeof(unsigned long long) * 4 * kMaxResidentWGs);
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

}  // namespace
