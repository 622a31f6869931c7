// Block-diagonal product for a general split structure (variable partitions of Section 3.1).
#pragma once
#include "dn_common.h"

namespace dn {

// ---------------------------------------------------------------------------------------------
// Block-diagonal product for a general split structure (variable partitions of Section 3.1; Section 4.1).
// Layer m has ga = split[m-1] input groups and gb = split[m] output groups; partition (a, b) owns the weights
// from input group a to output group b (and, for a = 0, the biases of group b).  For each input group a the
// inner sums over t in that group are Q^{m,a} (one dense product each); per partition
//   r^{(a,b)}_i[u] = sum_{j in group b} P^m_i[u][j] q^{m,a,i}_j,     t^{m,a,i}_j = sum_u P^m_i[u][j] 2 r^{(a,b(j))}_i[u].
// jv_part_kernel / jtv_part_kernel are the general (two-pass) form (layers 1..L-2; block L-1 = A^L diag(sigma') is
// applied as dense products per partition around them), jv_jtv_fused_part_kernel the single-pass one for small
// outputs, which streams all hidden layers' blocks.
struct PartArgs {
    int L, s, nL;
    int n[DN_MAX_LAYERS + 1];
    long long ld[DN_MAX_LAYERS + 1];
    int split[DN_MAX_LAYERS + 1];
    int bound[DN_MAX_LAYERS + 1][DN_MAX_SPLIT + 1];   // bound[m][k]: first neuron of group k of layer m
    int part_base[DN_MAX_LAYERS + 2];                 // first partition id of layer m (1..L)
    const float* P[DN_MAX_LAYERS + 1];                // P[m], m = 1..L-1
    const float* Qp[DN_MAX_LAYERS + 1];               // Q^{m,a}: Qp[m] + a * s * ld[m]
    float* Tp[DN_MAX_LAYERS + 1];                     // T^{m,a}: Tp[m] + a * s * ld[m]
    float* R;                                         // [partitions][s][ldr], hidden layers only
    long long ldr;
    // single-pass kernel: strip slot k is up to 256 columns of output group wgrp[k] of layer wlayer[k], starting
    // at column wcol[k] (a multiple of four)
    int nwslots;
    int wlayer[DN_MAX_WSLOTS];
    int wcol[DN_MAX_WSLOTS];
    int wgrp[DN_MAX_WSLOTS];
    int ga_max, gb_max;                               // largest split[m-1] and split[m] over the hidden layers m
    int m_hi;                                         // two-pass kernels: the stored blocks they stream are those of layers
                                                      // 1..m_hi (L-2: block L-1 is applied as dense products around them)
};

__device__ __forceinline__ int group_of(const int* bound, int groups, int j) {
    int g = 0;
#pragma unroll
    for (int k = 1; k < DN_MAX_SPLIT; ++k)
        if (k < groups && j >= bound[k]) g = k;
    return g;
}

// work-group = (sample, block of 8 outputs); each wave takes two rows u of every hidden layer's block
template <int RW>
__global__ __launch_bounds__(256) void jv_part_kernel(const PartArgs a, const unsigned* only_if) {
    // only_if (nullable): do nothing while that device word is zero (fall-back launch behind a single-pass kernel).
    // Virtual work-groups: walked with the grid as the stride, so a launch may have fewer work-groups.
    if (only_if && __hip_atomic_load(only_if, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == 0u) return;
    constexpr int UB = 4 * RW;              // rows per work-group: wave w takes rows u0 + w + 4 k, k < RW, together
    const int ublocks = (a.nL + UB - 1) / UB;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
    const long long slab = (long long)a.s * a.ldr;
    for (int vb = blockIdx.x; vb < a.s * ublocks; vb += gridDim.x) {
    const int i = vb / ublocks;
    const int u0 = (vb - i * ublocks) * UB;
    if (u0 + wave >= a.nL) continue;
    int urow[RW];
#pragma unroll
    for (int k = 0; k < RW; ++k) urow[k] = u0 + wave + 4 * k;
    for (int m = 1; m <= a.m_hi; ++m) {
        const int ga = a.split[m - 1], gb = a.split[m];
        const float* __restrict__ prow[RW];
#pragma unroll
        for (int k = 0; k < RW; ++k)      // rows past n_L repeat the first one; their sums are not stored
            prow[k] = a.P[m] + ((long long)i * a.nL + (urow[k] < a.nL ? urow[k] : urow[0])) * a.ld[m];
        // one output group at a time: its columns [lo, hi) are contiguous, so the sums of the ga partitions
        // that share them need no per-column bookkeeping.  Four columns per lane and step (rows are 16-byte
        // aligned and padded to a multiple of 4 floats); a group boundary may fall inside such a group of
        // four, which is then read for both neighbours and masked.
        for (int y = 0; y < gb; ++y) {
            const int lo = a.bound[m][y], hi = a.bound[m][y + 1];
            double acc[RW][DN_MAX_SPLIT];
#pragma unroll
            for (int k = 0; k < RW; ++k)
#pragma unroll
                for (int x = 0; x < DN_MAX_SPLIT; ++x) acc[k][x] = 0.0;
            for (int c4 = (lo >> 2) + lane; 4 * c4 < hi; c4 += 64) {
                const int j = 4 * c4;
                float4 p4[RW];
#pragma unroll
                for (int k = 0; k < RW; ++k) p4[k] = load_stream4(prow[k] + j);
                if (j < lo || j + 3 >= hi) {
#pragma unroll
                    for (int k = 0; k < RW; ++k) {
                        if (j + 0 < lo || j + 0 >= hi) p4[k].x = 0.f;
                        if (j + 1 < lo || j + 1 >= hi) p4[k].y = 0.f;
                        if (j + 2 < lo || j + 2 >= hi) p4[k].z = 0.f;
                        if (j + 3 < lo || j + 3 >= hi) p4[k].w = 0.f;
                    }
                }
#pragma unroll
                for (int x = 0; x < DN_MAX_SPLIT; ++x) {
                    if (x < ga) {
                        float4 q4 = *reinterpret_cast<const float4*>(a.Qp[m] + ((long long)x * a.s + i) * a.ld[m] + j);
                        // the padding of Q holds no data: keep it out of the products (0 * NaN)
                        if (j + 3 >= a.n[m]) {
                            if (j + 1 >= a.n[m]) q4.y = 0.f;
                            if (j + 2 >= a.n[m]) q4.z = 0.f;
                            q4.w = 0.f;
                        }
#pragma unroll
                        for (int k = 0; k < RW; ++k)
                            acc[k][x] += ((double)p4[k].x * q4.x + (double)p4[k].y * q4.y) +
                                         ((double)p4[k].z * q4.z + (double)p4[k].w * q4.w);
                    }
                }
            }
#pragma unroll
            for (int x = 0; x < DN_MAX_SPLIT; ++x) {
                if (x < ga) {
                    float* r = a.R + (long long)(a.part_base[m] + x * gb + y) * slab + (long long)i * a.ldr;
#pragma unroll
                    for (int k = 0; k < RW; ++k) {
                        const double t = wave_sum_d(acc[k][x]);
                        if (lane == 0 && urow[k] < a.nL) r[urow[k]] = (float)t;
                    }
                }
            }
        }
    }
}
}

// work-group = (sample, layer, chunk of 1024 columns); four columns per thread.  Layer L: t^{L,a} = 2 q^{L,a}.
__device__ __forceinline__ void jtv_part_block(const PartArgs& a, int chunks_total, int vb, float* rbar) {
    // rbar: [ga][gb][nL] of this layer
    const int i = vb / chunks_total;
    int c = vb - i * chunks_total;
    int m = 1;
    for (; m <= a.m_hi; ++m) {
        const int cm = (a.n[m] + 1023) >> 10;
        if (c < cm) break;
        c -= cm;
    }
    if (m > a.m_hi) m = a.L;          // the chunk after the streamed layers: the output layer
    const int ga = a.split[m - 1];
    if (m == a.L) {
        // identity block: groups of outputs stay apart by themselves
        for (int x = 0; x < ga; ++x)
            for (int u = threadIdx.x; u < a.nL; u += 256) {
                const long long e = ((long long)x * a.s + i) * a.ld[m] + u;
                a.Tp[m][e] = 2.0f * a.Qp[m][e];
            }
        return;
    }
    const int gb = a.split[m];
    const long long slab = (long long)a.s * a.ldr;
    for (int e = threadIdx.x; e < ga * gb * a.nL; e += 256) {
        const int pl = e / a.nL, u = e - pl * a.nL;
        rbar[e] = 2.0f * a.R[(long long)(a.part_base[m] + pl) * slab + (long long)i * a.ldr + u];
    }
    __syncthreads();
    const int j = (c << 10) + 4 * threadIdx.x;
    if (j >= a.n[m]) return;
    // output group of each of the four columns (columns past n_m: the last group; their sums are never stored)
    int bj[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) bj[e] = group_of(a.bound[m], gb, min(j + e, a.n[m] - 1));
    const bool one_group = bj[0] == bj[3];
    const float* __restrict__ pcol = a.P[m] + (long long)i * a.nL * a.ld[m] + j;
    double acc[DN_MAX_SPLIT][4];
#pragma unroll
    for (int x = 0; x < DN_MAX_SPLIT; ++x)
#pragma unroll
        for (int e = 0; e < 4; ++e) acc[x][e] = 0.0;
    // rows are padded to a multiple of 4 floats, so a full float4 is always readable
    if (one_group) {
#pragma unroll 4
        for (int u = 0; u < a.nL; ++u) {
            const float4 p4 = load_stream4(pcol + (long long)u * a.ld[m]);
#pragma unroll
            for (int x = 0; x < DN_MAX_SPLIT; ++x)
                if (x < ga) {
                    const double w = (double)rbar[(x * gb + bj[0]) * a.nL + u];
                    acc[x][0] += p4.x * w; acc[x][1] += p4.y * w; acc[x][2] += p4.z * w; acc[x][3] += p4.w * w;
                }
        }
    } else {
        for (int u = 0; u < a.nL; ++u) {
            const float4 p4 = load_stream4(pcol + (long long)u * a.ld[m]);
            const float pe[4] = {p4.x, p4.y, p4.z, p4.w};
#pragma unroll
            for (int x = 0; x < DN_MAX_SPLIT; ++x)
                if (x < ga) {
#pragma unroll
                    for (int e = 0; e < 4; ++e) acc[x][e] += (double)pe[e] * (double)rbar[(x * gb + bj[e]) * a.nL + u];
                }
        }
    }
#pragma unroll
    for (int x = 0; x < DN_MAX_SPLIT; ++x)
        if (x < ga) {
            float* t = a.Tp[m] + ((long long)x * a.s + i) * a.ld[m] + j;
            if (j + 3 < a.n[m]) {
                *reinterpret_cast<float4*>(t) = make_float4((float)acc[x][0], (float)acc[x][1], (float)acc[x][2], (float)acc[x][3]);
            } else {
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    if (j + e < a.n[m]) t[e] = (float)acc[x][e];
            }
        }
}

// virtual work-groups and only_if as in jv_part_kernel
__global__ __launch_bounds__(256) void jtv_part_kernel(const PartArgs a, int chunks_total, const unsigned* only_if) {
    extern __shared__ float rbar[];
    if (only_if && __hip_atomic_load(only_if, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == 0u) return;
    for (int vb = blockIdx.x; vb < a.s * chunks_total; vb += gridDim.x) {
        jtv_part_block(a, chunks_total, vb, rbar);
        __syncthreads();        // rbar is filled again by the next virtual work-group
    }
}

// Both passes in one for a split structure when n_L <= NLMAX and the hidden widths fit one work-group: the
// strips of P^m_i stay in registers as in jv_jtv_fused_kernel.  A strip slot is up to 256 columns of ONE output
// group of one layer (it starts at the multiple of four at or below the group's first column; columns outside
// the group are masked), so the sums of a wave belong to one partition per input group x and need no per-column
// selection: the kernel is bound by vector instruction issue, not by memory, and per-column selects in a
// layer-wide strip made it 2.3 times slower than the kernel of the other modes.  One HBM read of the stored
// blocks per product; all input groups go through each stage together (two barriers in all).
// Dynamic LDS: part[slot][x][u] (nwslots * ga_max * NLMAX floats), then rb[layer-1][x][y][u].
template <int NLMAX, int CH>
__global__ __launch_bounds__(1024) void jv_jtv_fused_part_kernel(const PartArgs a) {
    extern __shared__ float part_lds[];
    const int gx = a.ga_max, gy = a.gb_max;
    float* part = part_lds;
    float* rb = part_lds + a.nwslots * gx * NLMAX;
    const int i = blockIdx.x;
    // the wave index as a scalar: everything looked up by strip slot (layer, row stride, base pointers) then
    // stays in scalar registers instead of being recomputed per lane
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
    const int nwaves = blockDim.x >> 6;
    int m[CH], j[CH], yg[CH];
    bool live[CH], ok[CH][4];
    float4 p[CH][NLMAX];
#pragma unroll
    for (int ch = 0; ch < CH; ++ch) {
        const int slot = wave + ch * nwaves;
        const bool have = slot < a.nwslots;
        m[ch] = have ? a.wlayer[slot] : 1;
        yg[ch] = have ? a.wgrp[slot] : 0;
        j[ch] = have ? a.wcol[slot] + 4 * lane : 0;
        const int lo = a.bound[m[ch]][yg[ch]], hi = a.bound[m[ch]][yg[ch] + 1];
        live[ch] = have && j[ch] < hi;
#pragma unroll
        for (int e = 0; e < 4; ++e) ok[ch][e] = live[ch] && j[ch] + e >= lo && j[ch] + e < hi;
        const long long ldm = a.ld[m[ch]];
        const float* __restrict__ pbase = a.P[m[ch]] + (long long)i * a.nL * ldm + j[ch];
#pragma unroll
        for (int u = 0; u < NLMAX; ++u) {
            p[ch][u] = make_float4(0.f, 0.f, 0.f, 0.f);
            // rows are padded to a multiple of four floats: the whole group of four is readable
            if (live[ch] && u < a.nL) p[ch][u] = *reinterpret_cast<const float4*>(pbase + (long long)u * ldm);
        }
        if (!(ok[ch][0] && ok[ch][1] && ok[ch][2] && ok[ch][3])) {
            // columns of a neighbouring group, or padding: out of the sums
#pragma unroll
            for (int u = 0; u < NLMAX; ++u) {
                if (!ok[ch][0]) p[ch][u].x = 0.f;
                if (!ok[ch][1]) p[ch][u].y = 0.f;
                if (!ok[ch][2]) p[ch][u].z = 0.f;
                if (!ok[ch][3]) p[ch][u].w = 0.f;
            }
        }
    }
    // output layer (identity block): t^{L,x} = 2 q^{L,x}
    for (int x = 0; x < a.split[a.L - 1]; ++x)
        for (int u = threadIdx.x; u < a.nL; u += blockDim.x) {
            const long long e = ((long long)x * a.s + i) * a.ld[a.L] + u;
            a.Tp[a.L][e] = 2.0f * a.Qp[a.L][e];
        }
    // ---- partial sums of the strip for every input group x ---------------------------------------------
#pragma unroll
    for (int ch = 0; ch < CH; ++ch) {
        const int slot = wave + ch * nwaves;
        if (slot < a.nwslots) {                         // uniform in the wave
            const int ga = a.split[m[ch] - 1];
            for (int x = 0; x < ga; ++x) {
                float4 q4 = make_float4(0.f, 0.f, 0.f, 0.f);
                if (live[ch])
                    q4 = *reinterpret_cast<const float4*>(a.Qp[m[ch]] + ((long long)x * a.s + i) * a.ld[m[ch]] + j[ch]);
                // padding columns of Q are never written (and the masked P is zero there: keep 0 * NaN out)
                if (!ok[ch][0]) q4.x = 0.f;
                if (!ok[ch][1]) q4.y = 0.f;
                if (!ok[ch][2]) q4.z = 0.f;
                if (!ok[ch][3]) q4.w = 0.f;
                float* dst = part + (slot * gx + x) * NLMAX;
#pragma unroll
                for (int u = 0; u < NLMAX; ++u) {
                    if (u < a.nL) {
                        float v = (p[ch][u].x * q4.x + p[ch][u].y * q4.y) + (p[ch][u].z * q4.z + p[ch][u].w * q4.w);
                        v = wave_sum_to_lane63(v);
                        if (lane == 63) dst[u] = v;
                    }
                }
            }
        }
    }
    __syncthreads();
    // ---- r of every partition (layer, x, y), doubled: B = 2I ------------------------------------------
    for (int e = threadIdx.x; e < (a.L - 1) * gx * gy * NLMAX; e += blockDim.x) {
        const int u = e % NLMAX, y = (e / NLMAX) % gy, x = (e / (NLMAX * gy)) % gx, mm = e / (NLMAX * gy * gx) + 1;
        float rsum = 0.f;
        if (u < a.nL && x < a.split[mm - 1] && y < a.split[mm])
            for (int w = 0; w < a.nwslots; ++w)
                if (a.wlayer[w] == mm && a.wgrp[w] == y) rsum += part[(w * gx + x) * NLMAX + u];
        rb[e] = 2.0f * rsum;
    }
    __syncthreads();
    // ---- transposed product with the r of the strip's own partition -------------------------------------
#pragma unroll
    for (int ch = 0; ch < CH; ++ch) {
        if (live[ch]) {
            const int ga = a.split[m[ch] - 1];
            const bool whole = ok[ch][0] && ok[ch][1] && ok[ch][2] && ok[ch][3];
            for (int x = 0; x < ga; ++x) {
                const float* rx = rb + ((((m[ch] - 1) * gx + x) * gy) + yg[ch]) * NLMAX;
                float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
                for (int u = 0; u < NLMAX; ++u) {
                    if (u < a.nL) {
                        const float w0 = rx[u];
                        acc.x += p[ch][u].x * w0; acc.y += p[ch][u].y * w0; acc.z += p[ch][u].z * w0; acc.w += p[ch][u].w * w0;
                    }
                }
                float* t = a.Tp[m[ch]] + ((long long)x * a.s + i) * a.ld[m[ch]] + j[ch];
                if (whole) {
                    *reinterpret_cast<float4*>(t) = acc;
                } else {
                    // a group boundary inside these four columns: the neighbouring strip writes the others
                    if (ok[ch][0]) t[0] = acc.x;
                    if (ok[ch][1]) t[1] = acc.y;
                    if (ok[ch][2]) t[2] = acc.z;
                    if (ok[ch][3]) t[3] = acc.w;
                }
            }
        }
    }
}

// bias part of the sums over samples for a split structure: the biases of layer m belong to the partitions of
// input group 0, so their sums are the column sums of T^{m,0}.  K-slice k of the samples puts its sum into
// column n_{m-1} of slice k of the partial buffer, where the products with a column of ones put theirs in
// the other modes.  Work-group = (layer, 16 neurons, K-slice); 16 threads per neuron share the samples.
struct BiasSumArgs {
    int L, s;
    int n[DN_MAX_LAYERS + 1];
    long long ld[DN_MAX_LAYERS + 1];
    const float* T0[DN_MAX_LAYERS + 1];     // T^{m,0}
    float* W[DN_MAX_LAYERS + 1];            // partial buffer of layer m: [splits][n_m][ldw]
    long long ldw[DN_MAX_LAYERS + 1];
    long long slice[DN_MAX_LAYERS + 1];     // floats between the K-slices of layer m
    int splits, k_per_split;
    int first[DN_MAX_LAYERS + 2];           // first 16-neuron chunk of layer m
};

__global__ __launch_bounds__(256) void bias_colsum_kernel(const BiasSumArgs a) {
    __shared__ double red[16][17];
    const int chunk = blockIdx.x / a.splits, sidx = blockIdx.x - chunk * a.splits;
    int m = 1;
    for (int k = 2; k <= a.L; ++k)
        if (chunk >= a.first[k]) m = k;
    const int c = threadIdx.x & 15, r = threadIdx.x >> 4;
    const int j = (chunk - a.first[m]) * 16 + c;
    const int i_lo = sidx * a.k_per_split, i_hi = min(a.s, i_lo + a.k_per_split);
    double acc = 0.0;
    if (j < a.n[m]) {
        // eight loads in flight per thread, four partial chains, fixed order
        const float* __restrict__ col = a.T0[m] + j;
        const long long st = 16 * a.ld[m];
        double a0 = 0.0, a1 = 0.0, a2 = 0.0, a3 = 0.0;
        int i = i_lo + r;
        for (; i + 7 * 16 < i_hi; i += 8 * 16) {
            const float* p = col + (long long)i * a.ld[m];
            const float v0 = p[0], v1 = p[st], v2 = p[2 * st], v3 = p[3 * st];
            const float v4 = p[4 * st], v5 = p[5 * st], v6 = p[6 * st], v7 = p[7 * st];
            a0 += (double)v0 + (double)v4; a1 += (double)v1 + (double)v5;
            a2 += (double)v2 + (double)v6; a3 += (double)v3 + (double)v7;
        }
        for (; i < i_hi; i += 16) a0 += (double)col[(long long)i * a.ld[m]];
        acc = (a0 + a1) + (a2 + a3);
    }
    red[r][c] = acc;
    __syncthreads();
    if (r == 0 && j < a.n[m]) {
        double t = 0.0;
#pragma unroll
        for (int k = 0; k < 16; ++k) t += red[k][c];
        a.W[m][(long long)sidx * a.slice[m] + (long long)j * a.ldw[m] + a.n[m - 1]] = (float)t;
    }
}

// dst[k] = src[perm[k]]  (gather)  /  dst[perm[k]] = src[k]  (scatter);  perm lists the theta indices
// partition by partition, so that every partition is contiguous in the gathered order
__global__ __launch_bounds__(256) void perm_gather_kernel(const float* __restrict__ src, const int* __restrict__ perm,
                                                          float* __restrict__ dst, long long n, float scale) {
    for (long long e = (long long)blockIdx.x * 256 + threadIdx.x; e < n; e += (long long)gridDim.x * 256)
        dst[e] = scale * src[perm[e]];
}
__global__ __launch_bounds__(256) void perm_scatter_kernel(const float* __restrict__ src, const int* __restrict__ perm,
                                                           float* __restrict__ dst, long long n) {
    for (long long e = (long long)blockIdx.x * 256 + threadIdx.x; e < n; e += (long long)gridDim.x * 256)
        dst[perm[e]] = src[e];
}

}  // namespace dn
