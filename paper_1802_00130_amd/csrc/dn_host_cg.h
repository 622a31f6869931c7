// Conjugate gradient driver (Sections 2.2, 4.1, 4.3): launches and the host-side stopping logic.
// Part of the one translation unit dn_lib.hip (helpers live in its unnamed namespace).
#pragma once
#include "dn_host_product.h"

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
    if (part && active) {
        // p_0 in the theta layout; afterwards every update of p writes both layouts
        hipLaunchKernelGGL(perm_scatter_kernel, dim3(vgrid), dim3(256), 0, c->stream, p, perm, c->fptr(c->o_ptheta),
                           c->n);
        DN_HIP(c, hipGetLastError());
    }
    while (iters < max_iter && active) {
        int rc;
        if (part) {
            // the result stays in the theta layout; the inner-product kernel below fetches it through perm
            rc = gn_matvec(c, c->fptr(c->o_ptheta), c->fptr(c->o_qtheta), mode);
            if (rc != DN_OK) return rc;
        } else {
            // the fold at the end of the product also leaves the partial sums of p^T (G + lambda I) p
            rc = gn_matvec(c, p, q, mode, part1, (float)lambda);
            if (rc != DN_OK) return rc;
        }
        const CgState* cur = st + (iters & 1);
        CgState* nxt = st + ((iters + 1) & 1);
        {
            ProfScope ps(c, KC_CG_VEC);
            DN_HIP(c, ps.err);
            if (part) {
                hipLaunchKernelGGL(cg_dot_gather_kernel, dim3(grid), dim3(256), 0, c->stream, sg, p, q, (float)lambda,
                                   part1, perm, c->fptr(c->o_qtheta));
                DN_HIP(c, hipGetLastError());
            }
            hipLaunchKernelGGL(cg_update_dr_kernel, dim3(grid), dim3(256), 0, c->stream, sg, cur, part1, p, q,
                               (float)lambda, d_cg, r, part2);
            DN_HIP(c, hipGetLastError());
            if (part)
                hipLaunchKernelGGL(cg_update_p_kernel<true>, dim3(grid), dim3(256), 0, c->stream, sg, cur, nxt, part2,
                                   sigma * sigma, r, p, perm, c->fptr(c->o_ptheta));
            else
                hipLaunchKernelGGL(cg_update_p_kernel<false>, dim3(grid), dim3(256), 0, c->stream, sg, cur, nxt, part2,
                                   sigma * sigma, r, p, (const int*)nullptr, (float*)nullptr);
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
    return band_status(c);
}

}  // namespace
