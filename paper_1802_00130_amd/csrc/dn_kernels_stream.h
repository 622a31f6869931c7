// The two products with the stored Jacobian blocks P^m_i = d z^{L,i} / d s^{m,i} (Section 4.2): two-pass
// kernels and the single-pass kernel for small outputs.
#pragma once
#include "dn_common.h"

namespace dn {

// ---------------------------------------------------------------------------------------------
// Per-layer description of the stored blocks and product temporaries for the subsample.
struct StreamArgs {
    int L;              // weight layers
    int s;              // |S|
    int nL;             // output width
    int blockdiag;      // 0 full, 1 per-layer
    int n[DN_MAX_LAYERS + 1];            // n_0..n_L
    long long ld[DN_MAX_LAYERS + 1];     // row stride of Z/Q/T/P rows of layer m
    const float* P[DN_MAX_LAYERS + 1];   // P[m], m = 1..L-1: [s][nL][ld[m]]
    const float* Q[DN_MAX_LAYERS + 1];   // Q[m], m = 1..L: [s][ld[m]]
    const float* Qb[DN_MAX_LAYERS + 1];  // nullable: second half of a Q[m] whose sum over t was cut in two (fused kernel only)
    float* T[DN_MAX_LAYERS + 1];         // T[m], m = 1..L: [s][ld[m]]
    float* R;                            // [L][s][ldr] (full mode uses slot 0 only)
    long long ldr;
    // Two-pass kernels only: the block of the last hidden layer is not streamed from memory.  Since
    // P^{L-1}_i = A^L diag(sigma'(s^{L-1,i})) (Section 3.3 recursion applied once to the identity), its
    // two products are small dense products with A^L, done by the GEMM engine around these kernels.
    // fused kernel: wave w of a work-group owns float4 columns 64*wcol[w] + lane of layer wlayer[w]
    int nwslots;
    int wlayer[DN_MAX_WSLOTS];
    int wcol[DN_MAX_WSLOTS];
};

// J v, outer sum of Section 4.2: for sample i and output u,
//   full:       r_i[u]   = q^{L,i}_u + sum_{m<L} sum_j P^m_i[u][j] q^{m,i}_j
//   per-layer:  r^m_i[u] =                      sum_j P^m_i[u][j] q^{m,i}_j   (m < L),  r^L_i = q^{L,i}
// This kernel handles the stored blocks m <= L-2.  The block m = L-1 is applied before it as a small
// dense product (A^L times sigma'-scaled q^{L-1}), whose result is already inside Q[L] (full) or in
// slab L-2 of R (per-layer).
// Work-group = (sample, block of UB outputs); each wave reduces whole rows of P.
// Virtual work-groups: the kernel walks over them with its grid as the stride, so a launch may have fewer
// work-groups than there are.
// only_if (nullable): a device word; the kernel does nothing while it is zero (the launch is then the fall-back
// of a single-pass kernel that raises the word when it could not finish, made with a small grid).
template <int UB>
__global__ __launch_bounds__(256) void jv_rows_kernel(const StreamArgs a, const unsigned* only_if) {
    if (only_if && __hip_atomic_load(only_if, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == 0u) return;
    const int ublocks = (a.nL + UB - 1) / UB;
    for (int vb = blockIdx.x; vb < a.s * ublocks; vb += gridDim.x) {
    const int i = vb / ublocks;
    const int u0 = (vb - i * ublocks) * UB;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
    const long long slab = (long long)a.s * a.ldr;
    for (int uu = wave; uu < UB; uu += 4) {
        const int u = u0 + uu;
        if (u >= a.nL) break;
        // the pass is bound by HBM, so the sums are carried in fp64 at no cost in time
        double tot = 0.0;
        for (int m = 1; m + 1 < a.L; ++m) {
            const int nm4 = a.n[m] >> 2;
            const float* __restrict__ prow = a.P[m] + ((long long)i * a.nL + u) * a.ld[m];
            const float* __restrict__ q = a.Q[m] + (long long)i * a.ld[m];
            double acc = 0.0;
#pragma unroll 4
            for (int c = lane; c < nm4; c += 64) {
                const float4 p4 = load_stream4(prow + 4 * c);
                const float4 q4 = *reinterpret_cast<const float4*>(q + 4 * c);
                acc += ((double)p4.x * q4.x + (double)p4.y * q4.y) + ((double)p4.z * q4.z + (double)p4.w * q4.w);
            }
            const int tail = a.n[m] & 3;
            if (lane < tail) acc += (double)prow[4 * nm4 + lane] * q[4 * nm4 + lane];
            acc = wave_sum_d(acc);
            if (a.blockdiag) {
                if (lane == 0) a.R[(long long)(m - 1) * slab + (long long)i * a.ldr + u] = (float)acc;
            } else {
                tot += acc;
            }
        }
        if (lane == 0) {
            const float qL = a.Q[a.L][(long long)i * a.ld[a.L] + u];
            if (a.blockdiag) a.R[(long long)(a.L - 1) * slab + (long long)i * a.ldr + u] = qL;
            else             a.R[(long long)i * a.ldr + u] = (float)((double)qL + tot);
        }
    }
    }
}

// J^T, inner sum of Section 4.2 with B = 2I:  t^{m,i}_j = sum_u P^m_i[u][j] * 2 r_i[u]  (m < L),
// t^{L,i} = 2 r_i.  Stored blocks m <= L-2 and the output layer; t^{L-1} is a small dense product
// done after this kernel.  Work-group = (sample, layer, chunk of 1024 columns); threads own 4 columns.
__device__ __forceinline__ void jtv_cols_block(const StreamArgs& a, int chunks_total, int vb, float* rbar) {
    // decode (sample, layer, chunk): chunk list is layer-major within a sample
    const int i = vb / chunks_total;
    int c = vb - i * chunks_total;
    int m = 1;
    for (; m + 1 < a.L; ++m) {
        const int cm = (a.n[m] + 1023) >> 10;
        if (c < cm) break;
        c -= cm;
    }
    const long long slab = (long long)a.s * a.ldr;
    if (m + 1 >= a.L) {
        // output layer: identity block
        const float* r = a.R + (a.blockdiag ? (long long)(a.L - 1) * slab : 0) + (long long)i * a.ldr;
        for (int u = threadIdx.x; u < a.nL; u += 256) a.T[a.L][(long long)i * a.ld[a.L] + u] = 2.0f * r[u];
        return;
    }
    const float* r = a.R + (a.blockdiag ? (long long)(m - 1) * slab : 0) + (long long)i * a.ldr;
    for (int u = threadIdx.x; u < a.nL; u += 256) rbar[u] = 2.0f * r[u];
    __syncthreads();
    const int j = (c << 10) + 4 * threadIdx.x;
    if (j >= a.n[m]) return;
    const float* __restrict__ pcol = a.P[m] + (long long)i * a.nL * a.ld[m] + j;
    // HBM-bound pass: fp64 accumulators cost no time and keep the n_L-term sums exact to fp32
    double ax = 0.0, ay = 0.0, az = 0.0, aw = 0.0;
    // rows are padded to a multiple of 4 floats, so a full float4 is always readable
#pragma unroll 8
    for (int u = 0; u < a.nL; ++u) {
        const float4 p4 = load_stream4(pcol + (long long)u * a.ld[m]);
        const double w = (double)rbar[u];
        ax += p4.x * w; ay += p4.y * w; az += p4.z * w; aw += p4.w * w;
    }
    float* t = a.T[m] + (long long)i * a.ld[m] + j;
    *reinterpret_cast<float4*>(t) = make_float4((float)ax, (float)ay, (float)az, (float)aw);
}

// virtual work-groups and only_if as in jv_rows_kernel
__global__ __launch_bounds__(256) void jtv_cols_kernel(const StreamArgs a, int chunks_total, const unsigned* only_if) {
    extern __shared__ float rbar[];
    if (only_if && __hip_atomic_load(only_if, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == 0u) return;
    for (int vb = blockIdx.x; vb < a.s * chunks_total; vb += gridDim.x) {
        jtv_cols_block(a, chunks_total, vb, rbar);
        __syncthreads();        // rbar is filled again by the next virtual work-group
    }
}

// Both passes in one when n_L <= NLMAX and the hidden widths fit one work-group (all hidden layers'
// blocks, including m = L-1, are read from memory here: measured, rebuilding the last one from A^L inside
// this kernel is slower than streaming it):
// one work-group per sample, wave w keeps the 4-column strips of P^m_i (all n_L rows) in
// registers, so every stored element is read from HBM exactly once per product.
template <int NLMAX, int CH>
__global__ __launch_bounds__(1024) void jv_jtv_fused_kernel(const StreamArgs a) {
    // wave w owns strip slots w, w + waves, ... (CH of them at most); a slot is 256 columns of one layer
    __shared__ float part[DN_MAX_WSLOTS][NLMAX];
    __shared__ float rb[DN_MAX_LAYERS][NLMAX];
    const int i = blockIdx.x;
    // the wave index as a scalar: everything looked up by strip slot (layer, row stride, base pointers) then
    // stays in scalar registers instead of being recomputed per lane
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
    const int nwaves = blockDim.x >> 6;
    int m[CH], j[CH];
    bool live[CH];
    float4 p[CH][NLMAX];
    float4 q4[CH];
#pragma unroll
    for (int ch = 0; ch < CH; ++ch) {
        const int slot = wave + ch * nwaves;
        const bool have = slot < a.nwslots;
        m[ch] = have ? a.wlayer[slot] : 1;
        j[ch] = have ? 4 * (64 * a.wcol[slot] + lane) : 0;
        live[ch] = have && j[ch] < a.n[m[ch]];
        const long long ldm = a.ld[m[ch]];
        q4[ch] = make_float4(0.f, 0.f, 0.f, 0.f);
        if (live[ch]) q4[ch] = *reinterpret_cast<const float4*>(a.Q[m[ch]] + (long long)i * ldm + j[ch]);
        if (live[ch] && a.Qb[m[ch]]) {
            const float4 qb = *reinterpret_cast<const float4*>(a.Qb[m[ch]] + (long long)i * ldm + j[ch]);
            q4[ch].x += qb.x; q4[ch].y += qb.y; q4[ch].z += qb.z; q4[ch].w += qb.w;
        }
        // Every lane loads NLMAX rows without predicates (the kernel is bound by instruction issue as much as by
        // memory): rows past n_L repeat the last one and are never used, lanes past the layer's width read the
        // strip's first columns and multiply them by q = 0.
        const float* __restrict__ pbase = a.P[m[ch]] + (long long)i * a.nL * ldm + (live[ch] ? j[ch] : 0);
#pragma unroll
        for (int u = 0; u < NLMAX; ++u)
            p[ch][u] = *reinterpret_cast<const float4*>(pbase + (long long)min(u, a.nL - 1) * ldm);
    }
#pragma unroll
    for (int ch = 0; ch < CH; ++ch) {
        // columns past n_m hold padding (never written): keep them out of the sums
        const int rem = live[ch] ? a.n[m[ch]] - j[ch] : 4;
        if (rem < 4) {
            q4[ch].w = 0.f; if (rem < 3) q4[ch].z = 0.f; if (rem < 2) q4[ch].y = 0.f;
#pragma unroll
            for (int u = 0; u < NLMAX; ++u) {
                p[ch][u].w = 0.f; if (rem < 3) p[ch][u].z = 0.f; if (rem < 2) p[ch][u].y = 0.f;
            }
        }
        const int slot = wave + ch * nwaves;
#pragma unroll
        for (int u = 0; u < NLMAX; ++u) {
            if (u < a.nL) {
                float x = p[ch][u].x * q4[ch].x + p[ch][u].y * q4[ch].y + p[ch][u].z * q4[ch].z + p[ch][u].w * q4[ch].w;
                x = wave_sum_to_lane63(x);
                if (lane == 63 && slot < a.nwslots) part[slot][u] = x;
            }
        }
    }
    __syncthreads();
    {
        // r (full) or r^m (per layer), doubled: B = 2I
        const int u = threadIdx.x % NLMAX;
        const int slot = threadIdx.x / NLMAX;
        if (u < a.nL) {
            const float qL = a.Q[a.L][(long long)i * a.ld[a.L] + u];
            if (!a.blockdiag) {
                if (slot == 0) {
                    float rsum = qL;
                    for (int w = 0; w < a.nwslots; ++w) rsum += part[w][u];
                    rb[0][u] = 2.0f * rsum;
                    a.T[a.L][(long long)i * a.ld[a.L] + u] = 2.0f * rsum;
                }
            } else if (slot < a.L) {
                const int mm = slot + 1;
                if (mm == a.L) {
                    a.T[a.L][(long long)i * a.ld[a.L] + u] = 2.0f * qL;
                } else {
                    float rsum = 0.f;
                    for (int w = 0; w < a.nwslots; ++w)
                        if (a.wlayer[w] == mm) rsum += part[w][u];
                    rb[mm][u] = 2.0f * rsum;
                }
            }
        }
    }
    __syncthreads();
#pragma unroll
    for (int ch = 0; ch < CH; ++ch) {
        if (live[ch]) {
            const float* rr = a.blockdiag ? rb[m[ch]] : rb[0];
            float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
            for (int u = 0; u < NLMAX; ++u) {
                if (u < a.nL) {
                    const float w = rr[u];
                    acc.x += p[ch][u].x * w; acc.y += p[ch][u].y * w; acc.z += p[ch][u].z * w; acc.w += p[ch][u].w * w;
                }
            }
            *reinterpret_cast<float4*>(a.T[m[ch]] + (long long)i * a.ld[m[ch]] + j[ch]) = acc;
        }
    }
}

}  // namespace dn
