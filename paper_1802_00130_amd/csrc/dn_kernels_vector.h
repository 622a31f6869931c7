// Kernels over n-vectors in the theta layout: the fold of the sums over samples, the conjugate gradient
// updates, and the vector work of the outer Newton iteration.
#pragma once
#include "dn_common.h"

namespace dn {

// ---------------------------------------------------------------------------------------------
// Final step of every sum over samples: fold the K-slices of the T^T [Z, 1] contraction and add
// the regularisation term (Section 2.2 gradient; Section 4.3 product):
//   out[e] = x[e] / C + scale * sum_slices W[slice][j][t]
// e walks the theta layout; column t = n_{m-1} of W holds the bias sums.
struct ReduceArgs {
    int L;
    int n[DN_MAX_LAYERS + 1];
    long long off[DN_MAX_LAYERS + 1];   // theta offset of layer m's weights (m = 1..L); biases follow them
    const float* W[DN_MAX_LAYERS + 1];  // W[m]: [splits][n_m][ldw[m]]
    long long ldw[DN_MAX_LAYERS + 1];
    long long split_stride[DN_MAX_LAYERS + 1];
    int splits[DN_MAX_LAYERS + 1];
    int blk_begin[DN_MAX_LAYERS + 2];   // first work-group of layer m; its work-groups share the layer's items
    int items[DN_MAX_LAYERS + 1];       // items of layer m; one item = (row j, 1024 columns)
    int chunks[DN_MAX_LAYERS + 1];      // 1024-column chunks per row of layer m
};

typedef float f32x4v __attribute__((ext_vector_type(4), aligned(4)));

// dot (nullable): partial sums of x^T (out + lambda x) per work-group, in fp64; the work-groups of layer m are
// [blk_begin[m], blk_begin[m+1]), so a conjugate gradient step whose product ends here gets p^T (G + lambda I) p
// (whole, or per layer) without another pass over the two vectors.
__global__ __launch_bounds__(256) void tn_reduce_kernel(const ReduceArgs a, const float* __restrict__ x,
                                                        float* __restrict__ out, float invC, float scale,
                                                        double* __restrict__ dot, float lambda) {
    __shared__ double red[4];
    int m = 1;
#pragma unroll
    for (int k = 2; k <= DN_MAX_LAYERS; ++k)
        if (k <= a.L && (int)blockIdx.x >= a.blk_begin[k]) m = k;
    const int nb = a.blk_begin[m + 1] - a.blk_begin[m];
    const int np = a.n[m - 1];
    const long long ss = a.split_stride[m];
    const int ns = a.splits[m];
    double dacc = 0.0;
    for (int item = (int)blockIdx.x - a.blk_begin[m]; item < a.items[m]; item += nb) {
        const int j = item / a.chunks[m];
        const int t = (item - j * a.chunks[m]) * 1024 + 4 * (int)threadIdx.x;
        if (t > np) continue;                     // columns 0..np (np = bias column)
        const float* __restrict__ w = a.W[m] + (long long)j * a.ldw[m] + t;   // 16-byte aligned: ldw % 4 == 0
        // fixed summation order: slices in increasing order, four partial chains
        float4 acc0 = make_float4(0.f, 0.f, 0.f, 0.f), acc1 = acc0, acc2 = acc0, acc3 = acc0;
        int sidx = 0;
        for (; sidx + 4 <= ns; sidx += 4) {
            const float4 w0 = *reinterpret_cast<const float4*>(w + (long long)(sidx + 0) * ss);
            const float4 w1 = *reinterpret_cast<const float4*>(w + (long long)(sidx + 1) * ss);
            const float4 w2 = *reinterpret_cast<const float4*>(w + (long long)(sidx + 2) * ss);
            const float4 w3 = *reinterpret_cast<const float4*>(w + (long long)(sidx + 3) * ss);
            acc0.x += w0.x; acc0.y += w0.y; acc0.z += w0.z; acc0.w += w0.w;
            acc1.x += w1.x; acc1.y += w1.y; acc1.z += w1.z; acc1.w += w1.w;
            acc2.x += w2.x; acc2.y += w2.y; acc2.z += w2.z; acc2.w += w2.w;
            acc3.x += w3.x; acc3.y += w3.y; acc3.z += w3.z; acc3.w += w3.w;
        }
        for (; sidx < ns; ++sidx) {
            const float4 w0 = *reinterpret_cast<const float4*>(w + (long long)sidx * ss);
            acc0.x += w0.x; acc0.y += w0.y; acc0.z += w0.z; acc0.w += w0.w;
        }
        float s4[4] = {(acc0.x + acc1.x) + (acc2.x + acc3.x), (acc0.y + acc1.y) + (acc2.y + acc3.y),
                       (acc0.z + acc1.z) + (acc2.z + acc3.z), (acc0.w + acc1.w) + (acc2.w + acc3.w)};
        const long long wbase = a.off[m] + (long long)j * np;                // weight (j, t) sits at wbase + t
        const long long bidx = a.off[m] + (long long)np * a.n[m] + j;        // bias j
        if (t + 3 < np) {
            const f32x4v xv = *reinterpret_cast<const f32x4v*>(x + wbase + t);
            f32x4v o;
#pragma unroll
            for (int c = 0; c < 4; ++c) o[c] = xv[c] * invC + scale * s4[c];
            *reinterpret_cast<f32x4v*>(out + wbase + t) = o;
            if (dot) {
                double d4[4];
#pragma unroll
                for (int c = 0; c < 4; ++c) d4[c] = (double)xv[c] * (double)(o[c] + lambda * xv[c]);
                dacc += (d4[0] + d4[1]) + (d4[2] + d4[3]);
            }
        } else {
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                const int tt = t + c;
                if (tt <= np) {
                    const long long e = tt < np ? wbase + tt : bidx;
                    const float xe = x[e];
                    const float o = xe * invC + scale * s4[c];
                    out[e] = o;
                    if (dot) dacc += (double)xe * (double)(o + lambda * xe);
                }
            }
        }
    }
    if (dot) {
        dacc = block_sum_d(dacc, red);
        if (threadIdx.x == 0) dot[blockIdx.x] = dacc;
    }
}

// ---------------------------------------------------------------------------------------------
// Conjugate gradient vector kernels.  The n-vector is cut into segments (one for the full
// system, one per layer for the block-diagonal systems, Section 4.1); each segment is cut into
// chunks, one work-group per chunk; dot products are reduced in fp64 in a fixed order.
struct CgSegs {
    int nseg;
    int chunk;                           // elements per work-group
    long long off[DN_MAX_SEGS + 1];      // segment k covers [off[k], off[k+1])
    int cb[DN_MAX_SEGS + 1];             // first work-group of segment k; cb[nseg] = grid size
    int pb[DN_MAX_SEGS + 1];             // partial sums of p^T A p that belong to segment k: [pb[k], pb[k+1])
};

struct CgState {                         // lives in device memory, one per iteration parity
    double rho[DN_MAX_SEGS];             // r^T r
    double gnorm2[DN_MAX_SEGS];          // g^T g
    int active[DN_MAX_SEGS];
    int pad[DN_MAX_SEGS];
};

__device__ __forceinline__ void cg_locate(const CgSegs& sg, int& seg, long long& lo, long long& hi) {
    seg = 0;
    for (int k = 1; k < sg.nseg; ++k)
        if ((int)blockIdx.x >= sg.cb[k]) seg = k;
    lo = sg.off[seg] + (long long)((int)blockIdx.x - sg.cb[seg]) * sg.chunk;
    hi = lo + sg.chunk;
    if (hi > sg.off[seg + 1]) hi = sg.off[seg + 1];
}

// Elements [lo, hi) of a chunk: groups of four through 16-byte accesses (fv; the vectors carry no alignment
// beyond that of a float: segments start anywhere in theta), the last hi - lo mod 4 one by one (fs).
template <class FV, class FS>
__device__ __forceinline__ void cg_sweep(long long lo, long long hi, FV fv, FS fs) {
    const long long tail = lo + ((hi - lo) & ~3LL);
    for (long long e = lo + 4 * (long long)threadIdx.x; e < tail; e += 1024) fv(e);
    if (tail + threadIdx.x < hi) fs(tail + threadIdx.x);
}
__device__ __forceinline__ f32x4v ld4(const float* p) { return *reinterpret_cast<const f32x4v*>(p); }
__device__ __forceinline__ void st4(float* p, f32x4v v) { *reinterpret_cast<f32x4v*>(p) = v; }
// streaming variants for vectors that nothing reads again soon (no allocation in the caches)
__device__ __forceinline__ f32x4v ld4_stream(const float* p) { return __builtin_nontemporal_load(reinterpret_cast<const f32x4v*>(p)); }
__device__ __forceinline__ void st4_stream(float* p, f32x4v v) { __builtin_nontemporal_store(v, reinterpret_cast<f32x4v*>(p)); }

// d = 0, r = p = -g, partial g^T g
__global__ __launch_bounds__(256) void cg_init_kernel(const CgSegs sg, const float* __restrict__ g,
                                                      float* __restrict__ d, float* __restrict__ r,
                                                      float* __restrict__ p, double* __restrict__ partials) {
    __shared__ double red[4];
    int seg; long long lo, hi;
    cg_locate(sg, seg, lo, hi);
    double acc = 0.0;
    cg_sweep(lo, hi,
             [&](long long e) {
                 const f32x4v ge = ld4(g + e);
                 const f32x4v z = {0.f, 0.f, 0.f, 0.f};
                 st4(d + e, z); st4(r + e, -ge); st4(p + e, -ge);
                 acc += ((double)ge[0] * (double)ge[0] + (double)ge[1] * (double)ge[1]) +
                        ((double)ge[2] * (double)ge[2] + (double)ge[3] * (double)ge[3]);
             },
             [&](long long e) {
                 const float ge = g[e];
                 d[e] = 0.f; r[e] = -ge; p[e] = -ge;
                 acc += (double)ge * (double)ge;
             });
    acc = block_sum_d(acc, red);
    if (threadIdx.x == 0) partials[blockIdx.x] = acc;
}

__global__ __launch_bounds__(256) void cg_init_state_kernel(const CgSegs sg, const double* __restrict__ partials,
                                                            CgState* __restrict__ st) {
    __shared__ double red[4];
    for (int k = 0; k < sg.nseg; ++k) {
        const double gg = block_sum_range(partials, sg.cb[k], sg.cb[k + 1], red);
        if (threadIdx.x == 0) {
            st[0].rho[k] = gg; st[0].gnorm2[k] = gg; st[0].active[k] = gg > 0.0 ? 1 : 0;
            st[1].rho[k] = gg; st[1].gnorm2[k] = gg; st[1].active[k] = gg > 0.0 ? 1 : 0;
        }
    }
}

// Partitions only (the other modes take these partial sums from the fold of the product): partial
// p^T (q + lambda p), with q fetched from the product's result in the theta layout, q[e] = q_theta[perm[e]],
// and left in q for the update that follows.
__global__ __launch_bounds__(256) void cg_dot_gather_kernel(const CgSegs sg, const float* __restrict__ p,
                                                            float* __restrict__ q, float lambda,
                                                            double* __restrict__ partials,
                                                            const int* __restrict__ perm,
                                                            const float* __restrict__ q_theta) {
    __shared__ double red[4];
    int seg; long long lo, hi;
    cg_locate(sg, seg, lo, hi);
    double acc = 0.0;
    cg_sweep(lo, hi,
             [&](long long e) {
                 const f32x4v pe = ld4(p + e);
                 f32x4v qe;
#pragma unroll
                 for (int k = 0; k < 4; ++k) qe[k] = q_theta[perm[e + k]];
                 st4(q + e, qe);
                 double s4[4];
#pragma unroll
                 for (int k = 0; k < 4; ++k) s4[k] = (double)pe[k] * (double)(qe[k] + lambda * pe[k]);
                 acc += (s4[0] + s4[1]) + (s4[2] + s4[3]);
             },
             [&](long long e) {
                 const float pe = p[e], qe = q_theta[perm[e]];
                 q[e] = qe;
                 acc += (double)pe * (double)(qe + lambda * pe);
             });
    acc = block_sum_d(acc, red);
    if (threadIdx.x == 0) partials[blockIdx.x] = acc;
}

// alpha = rho / p^T A p;  d += alpha p;  r -= alpha (q + lambda p);  partial r^T r
__global__ __launch_bounds__(256) void cg_update_dr_kernel(const CgSegs sg, const CgState* __restrict__ st,
                                                           const double* __restrict__ pq_partials,
                                                           const float* __restrict__ p, const float* __restrict__ q,
                                                           float lambda, float* __restrict__ d, float* __restrict__ r,
                                                           double* __restrict__ rr_partials) {
    __shared__ double red[4];
    int seg; long long lo, hi;
    cg_locate(sg, seg, lo, hi);
    if (!st->active[seg]) {
        if (threadIdx.x == 0) rr_partials[blockIdx.x] = 0.0;
        return;
    }
    const double pq = block_sum_range(pq_partials, sg.pb[seg], sg.pb[seg + 1], red);
    const float alpha = (float)(st->rho[seg] / pq);
    double acc = 0.0;
    cg_sweep(lo, hi,
             [&](long long e) {
                 const f32x4v pe = ld4(p + e), qe = ld4_stream(q + e);
                 f32x4v de = ld4_stream(d + e), re = ld4(r + e);
                 double s4[4];
#pragma unroll
                 for (int k = 0; k < 4; ++k) {
                     de[k] += alpha * pe[k];
                     re[k] = re[k] - alpha * (qe[k] + lambda * pe[k]);
                     s4[k] = (double)re[k] * (double)re[k];
                 }
                 st4_stream(d + e, de); st4(r + e, re);
                 acc += (s4[0] + s4[1]) + (s4[2] + s4[3]);
             },
             [&](long long e) {
                 const float pe = p[e];
                 d[e] += alpha * pe;
                 const float re = r[e] - alpha * (q[e] + lambda * pe);
                 r[e] = re;
                 acc += (double)re * (double)re;
             });
    acc = block_sum_d(acc, red);
    if (threadIdx.x == 0) rr_partials[blockIdx.x] = acc;
}

// rho' = r^T r;  stop test ||r|| <= sigma ||g||;  beta = rho'/rho;  p = r + beta p.
// SCATTER: the new p also goes to p_theta[perm[e]], the theta layout the next product reads (a segment that has
// stopped writes nothing: its p, and with it p_theta, stay as they are).
template <bool SCATTER>
__global__ __launch_bounds__(256) void cg_update_p_kernel(const CgSegs sg, const CgState* __restrict__ st_cur,
                                                          CgState* __restrict__ st_next,
                                                          const double* __restrict__ rr_partials, double sigma2,
                                                          const float* __restrict__ r, float* __restrict__ p,
                                                          const int* __restrict__ perm, float* __restrict__ p_theta) {
    __shared__ double red[4];
    int seg; long long lo, hi;
    cg_locate(sg, seg, lo, hi);
    const bool first = ((int)blockIdx.x == sg.cb[seg]) && threadIdx.x == 0;
    if (!st_cur->active[seg]) {
        if (first) { st_next->rho[seg] = st_cur->rho[seg]; st_next->active[seg] = 0; }
        return;
    }
    const double rho_new = block_sum_range(rr_partials, sg.cb[seg], sg.cb[seg + 1], red);
    const bool stop = rho_new <= sigma2 * st_cur->gnorm2[seg];
    if (first) { st_next->rho[seg] = rho_new; st_next->active[seg] = stop ? 0 : 1; }
    if (stop) return;
    const float beta = (float)(rho_new / st_cur->rho[seg]);
    cg_sweep(lo, hi,
             [&](long long e) {
                 const f32x4v re = ld4(r + e);
                 f32x4v pe = ld4(p + e);
#pragma unroll
                 for (int k = 0; k < 4; ++k) pe[k] = re[k] + beta * pe[k];
                 st4(p + e, pe);
                 if (SCATTER) {
#pragma unroll
                     for (int k = 0; k < 4; ++k) p_theta[perm[e + k]] = pe[k];
                 }
             },
             [&](long long e) {
                 const float pe = r[e] + beta * p[e];
                 p[e] = pe;
                 if (SCATTER) p_theta[perm[e]] = pe;
             });
}

// ---------------------------------------------------------------------------------------------
// Outer Newton iteration (Section 4.3 direction combination, Section 4.5 line search): vector kernels.

// Partial sums of the five inner products of the two-variable system and of the step-size test:
//   0: g^T d   1: g^T db   2: d^T Gd   3: db^T Gd   4: db^T Gdb        partials[k * gridDim.x + block]
__global__ __launch_bounds__(256) void newton_dots_kernel(const float* __restrict__ g, const float* __restrict__ d,
                                                          const float* __restrict__ db,
                                                          const float* __restrict__ Gd,
                                                          const float* __restrict__ Gdb, long long n,
                                                          double* __restrict__ partials) {
    __shared__ double red[4];
    double a0 = 0.0, a1 = 0.0, a2 = 0.0, a3 = 0.0, a4 = 0.0;
    for (long long e = (long long)blockIdx.x * 256 + threadIdx.x; e < n; e += (long long)gridDim.x * 256) {
        const double ge = g[e], de = d[e], be = db[e], gd = Gd[e], gb = Gdb[e];
        a0 += ge * de; a1 += ge * be; a2 += de * gd; a3 += be * gd; a4 += be * gb;
    }
    const double v[5] = {a0, a1, a2, a3, a4};
#pragma unroll
    for (int k = 0; k < 5; ++k) {
        const double t = block_sum_d(v[k], red);
        if (threadIdx.x == 0) partials[(long long)k * gridDim.x + blockIdx.x] = t;
    }
}

// out[k] = sum of partials[k * nblocks .. (k+1) * nblocks), fixed order
__global__ __launch_bounds__(256) void newton_dots_finalize_kernel(const double* __restrict__ partials, int nblocks,
                                                                   double* __restrict__ out) {
    __shared__ double red[4];
    for (int k = 0; k < 5; ++k) {
        const double t = block_sum_range(partials, k * nblocks, (k + 1) * nblocks, red);
        if (threadIdx.x == 0) out[k] = t;
    }
}

// out = a x + b y   (out may alias x or y)
__global__ __launch_bounds__(256) void axpby_kernel(float a, const float* x, float b, const float* y, float* out,
                                                    long long n) {
    for (long long e = (long long)blockIdx.x * 256 + threadIdx.x; e < n; e += (long long)gridDim.x * 256)
        out[e] = a * x[e] + b * y[e];
}

}  // namespace dn
