// Streaming (HBM-bound) kernels of the path: the two passes over the stored Jacobian blocks
// P^m_i = d z^{L,i} / d s^{m,i}, their fused single-pass form, reductions and CG vector updates.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#define DN_MAX_LAYERS 8
#define DN_MAX_WSLOTS 32
#define DN_MAX_PARTIALS 1024
#define DN_MAX_SPLIT 4                                  // neuron groups per layer of a split structure
#define DN_MAX_SEGS (DN_MAX_LAYERS * DN_MAX_SPLIT * DN_MAX_SPLIT)   // independent CG systems (partitions)

namespace dn {

// DPP lane permutation inside rows of 16 lanes (no LDS traffic); CTRL as in the ISA:
// 0xB1 = quad_perm [1,0,3,2], 0x4E = quad_perm [2,3,0,1], 0x141 = row_half_mirror, 0x140 = row_mirror.
template <int CTRL>
__device__ __forceinline__ float dpp_move(float x) {
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), CTRL, 0xf, 0xf, false));
}

// Sum over the 64 lanes of a wave, result in lane 63 only, with DPP alone (no LDS traffic): rows of 16
// lanes first, then row_bcast:15 adds the sum of row r-1 into rows 1 and 3, then row_bcast:31 adds the
// sum of rows 0-1 into rows 2 and 3.
__device__ __forceinline__ float wave_sum_to_lane63(float x) {
    x += dpp_move<0xB1>(x);
    x += dpp_move<0x4E>(x);
    x += dpp_move<0x141>(x);
    x += dpp_move<0x140>(x);
    x += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0x142, 0xa, 0xf, false));
    x += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0x143, 0xc, 0xf, false));
    return x;
}

__device__ __forceinline__ double wave_sum_d(double x) {
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) x += __shfl_xor(x, o, 64);
    return x;
}

// Sum of one double per thread over a 256-thread work-group, same order every run.
// Result valid in every thread.
__device__ __forceinline__ double block_sum_d(double x, double* lds /* >= 4 doubles */) {
    x = wave_sum_d(x);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) lds[threadIdx.x >> 6] = x;
    __syncthreads();
    return (lds[0] + lds[1]) + (lds[2] + lds[3]);
}

// Sum partials[lo..hi) cooperatively (256 threads), fixed order.
__device__ __forceinline__ double block_sum_range(const double* __restrict__ partials, int lo, int hi, double* lds) {
    double x = 0.0;
    for (int i = lo + (int)threadIdx.x; i < hi; i += 256) x += partials[i];
    return block_sum_d(x, lds);
}

// ---------------------------------------------------------------------------------------------
// Row gather: XS[i][:] = X[S[i]][:]   (the subsample of Section 4.3)
__global__ __launch_bounds__(256) void gather_rows_kernel(const float* __restrict__ X, const int* __restrict__ S,
                                                          float* __restrict__ XS, int s, int n0, int l,
                                                          long long ldx, long long ldxs) {
    const long long total = (long long)s * n0;
    for (long long e = (long long)blockIdx.x * 256 + threadIdx.x; e < total; e += (long long)gridDim.x * 256) {
        const int i = (int)(e / n0);
        const int t = (int)(e - (long long)i * n0);
        const int row = min(max(S[i], 0), l - 1);  // ids outside [0, l) are clamped, never dereferenced
        XS[(long long)i * ldxs + t] = X[(long long)row * ldx + t];
    }
}

// ---------------------------------------------------------------------------------------------
// First stored block (Section 3.3, recursion started from dz^L/dz^L = I):
//   P^{L-1}_i[u][j] = w^L_{ju} * sigma'(s^{L-1,i}_j),   sigma' = z(1-z).
// AL is the padded copy of the n_L x n_{L-1} slice of theta for layer L.
__global__ __launch_bounds__(256) void jac_init_kernel(const float* __restrict__ AL, const float* __restrict__ Z,
                                                       float* __restrict__ P, int s, int nL, int nh, long long ld) {
    // AL, Z and P share the padded row length ld (a multiple of 4, rows 16-byte aligned); blockIdx.y walks the
    // samples, the x dimension the n_L x ld/4 groups of four columns of one sample
    const int ld4 = (int)(ld >> 2);
    const int total4 = nL * ld4;
    for (int i = blockIdx.y; i < s; i += gridDim.y) {
        const float* __restrict__ z = Z + (long long)i * ld;
        float* __restrict__ Pi = P + (long long)i * nL * ld;
        for (int e = blockIdx.x * 256 + threadIdx.x; e < total4; e += gridDim.x * 256) {
            const int u = e / ld4;
            const int j = 4 * (e - u * ld4);
            if (j >= nh) continue;                       // padding columns are never written
            const float4 a4 = *reinterpret_cast<const float4*>(AL + (long long)u * ld + j);
            const float4 z4 = *reinterpret_cast<const float4*>(z + j);
            const float4 o = make_float4(a4.x * (z4.x * (1.0f - z4.x)), a4.y * (z4.y * (1.0f - z4.y)),
                                         a4.z * (z4.z * (1.0f - z4.z)), a4.w * (z4.w * (1.0f - z4.w)));
            float* dst = Pi + (long long)u * ld + j;
            if (j + 3 < nh) {
                *reinterpret_cast<float4*>(dst) = o;
            } else {
                dst[0] = o.x;
                if (j + 1 < nh) dst[1] = o.y;
                if (j + 2 < nh) dst[2] = o.z;
            }
        }
    }
}

// Row copy into a padded layout: dst[r][c] = src[r][c], rows of src are dense.
__global__ __launch_bounds__(256) void pad_rows_kernel(const float* __restrict__ src, float* __restrict__ dst,
                                                       long long rows, int cols, long long ld) {
    const long long total = rows * cols;
    for (long long e = (long long)blockIdx.x * 256 + threadIdx.x; e < total; e += (long long)gridDim.x * 256) {
        const long long rr = e / cols;
        dst[rr * ld + (e - rr * cols)] = src[e];
    }
}

// dst[c][r] = src[r][c] for a dense rows x cols matrix (32x32 tiles through LDS).  Used to keep
// W^m (the transpose of the theta slice A^m) beside A^m, so that products with A^m as the right
// operand also read both operands K-contiguously.
__global__ __launch_bounds__(256) void transpose_kernel(const float* __restrict__ src, float* __restrict__ dst,
                                                        int rows, int cols) {
    __shared__ float tile[32][33];
    const int bx = blockIdx.x * 32, by = blockIdx.y * 32;
    const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;   // 32 x 8
#pragma unroll
    for (int k = 0; k < 32; k += 8) {
        const int rr = by + ty + k, cc = bx + tx;
        if (rr < rows && cc < cols) tile[ty + k][tx] = src[(long long)rr * cols + cc];
    }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < 32; k += 8) {
        const int cc = bx + ty + k, rr = by + tx;
        if (rr < rows && cc < cols) dst[(long long)cc * rows + rr] = tile[tx][ty + k];
    }
}

// Dense copy of a stored block (drops the row padding).
__global__ __launch_bounds__(256) void unpad_rows_kernel(const float* __restrict__ src, float* __restrict__ dst,
                                                         long long rows, int cols, long long ld) {
    const long long total = rows * cols;
    for (long long e = (long long)blockIdx.x * 256 + threadIdx.x; e < total; e += (long long)gridDim.x * 256) {
        const long long rr = e / cols;
        dst[e] = src[rr * ld + (e - rr * cols)];
    }
}

// ---------------------------------------------------------------------------------------------
// Loss partial sums: sum (z - y)^2 in fp64; optionally writes the back-propagation seed
// 2 (z^L - y)  (Section 3.4) and a dense copy of z^L.
// accumulate != 0: the partial sums are added to what an earlier chunk of the samples left there.
__global__ __launch_bounds__(256) void loss_delta_kernel(const float* __restrict__ ZL, long long ldz,
                                                         const float* __restrict__ Y, int l, int nL,
                                                         float* __restrict__ delta, long long ldd,
                                                         float* __restrict__ zl_out, double* __restrict__ partials,
                                                         int accumulate) {
    __shared__ double red[4];
    const long long total = (long long)l * nL;
    double acc = 0.0;
    for (long long e = (long long)blockIdx.x * 256 + threadIdx.x; e < total; e += (long long)gridDim.x * 256) {
        const long long i = e / nL;
        const int u = (int)(e - i * nL);
        const float z = ZL[i * ldz + u];
        const float dlt = z - Y[e];
        acc += (double)dlt * (double)dlt;
        if (delta) delta[i * ldd + u] = 2.0f * dlt;
        if (zl_out) zl_out[e] = z;
    }
    acc = block_sum_d(acc, red);
    if (threadIdx.x == 0) partials[blockIdx.x] = accumulate ? partials[blockIdx.x] + acc : acc;
}

__global__ __launch_bounds__(256) void sumsq_kernel(const float* __restrict__ x, long long n,
                                                    double* __restrict__ partials) {
    __shared__ double red[4];
    double acc = 0.0;
    for (long long e = (long long)blockIdx.x * 256 + threadIdx.x; e < n; e += (long long)gridDim.x * 256) {
        const double v = (double)x[e];
        acc += v * v;
    }
    acc = block_sum_d(acc, red);
    if (threadIdx.x == 0) partials[blockIdx.x] = acc;
}

// f = reg / (2C) + loss / l   (Section 2.1 objective)
__global__ __launch_bounds__(256) void objective_finalize_kernel(const double* __restrict__ loss_partials, int nloss,
                                                                 const double* __restrict__ reg_partials, int nreg,
                                                                 double inv2C, double invl, double* __restrict__ f) {
    __shared__ double red[4];
    const double a = block_sum_range(loss_partials, 0, nloss, red);
    const double b = block_sum_range(reg_partials, 0, nreg, red);
    if (threadIdx.x == 0) *f = b * inv2C + a * invl;
}

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
template <int UB>
__global__ __launch_bounds__(256) void jv_rows_kernel(const StreamArgs a) {
    const int ublocks = (a.nL + UB - 1) / UB;
    const int i = blockIdx.x / ublocks;
    const int u0 = (blockIdx.x - i * ublocks) * UB;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
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
                const float4 p4 = *reinterpret_cast<const float4*>(prow + 4 * c);
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

// J^T, inner sum of Section 4.2 with B = 2I:  t^{m,i}_j = sum_u P^m_i[u][j] * 2 r_i[u]  (m < L),
// t^{L,i} = 2 r_i.  Stored blocks m <= L-2 and the output layer; t^{L-1} is a small dense product
// done after this kernel.  Work-group = (sample, layer, chunk of 1024 columns); threads own 4 columns.
__global__ __launch_bounds__(256) void jtv_cols_kernel(const StreamArgs a, int chunks_total) {
    extern __shared__ float rbar[];
    // decode (sample, layer, chunk): chunk list is layer-major within a sample
    const int i = blockIdx.x / chunks_total;
    int c = blockIdx.x - i * chunks_total;
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
        const float4 p4 = *reinterpret_cast<const float4*>(pcol + (long long)u * a.ld[m]);
        const double w = (double)rbar[u];
        ax += p4.x * w; ay += p4.y * w; az += p4.z * w; aw += p4.w * w;
    }
    float* t = a.T[m] + (long long)i * a.ld[m] + j;
    *reinterpret_cast<float4*>(t) = make_float4((float)ax, (float)ay, (float)az, (float)aw);
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
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
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
        const float* __restrict__ pbase = a.P[m[ch]] + (long long)i * a.nL * ldm + j[ch];
#pragma unroll
        for (int u = 0; u < NLMAX; ++u) {
            p[ch][u] = make_float4(0.f, 0.f, 0.f, 0.f);
            if (live[ch] && u < a.nL) p[ch][u] = *reinterpret_cast<const float4*>(pbase + (long long)u * ldm);
        }
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

// ---------------------------------------------------------------------------------------------
// Single pass over the stored blocks for wide outputs (n_L > 16): teams of work-groups.
//
// The two products of Section 4.2 need every element of P^m_i twice, and r_i = J_i v must be complete
// before the transposed product can start.  One sample's blocks (n_L x sum n_m floats) exceed what one
// work-group can hold, so a TEAM of G work-groups shares a sample: work-group (rs, cs) keeps rows
// [rs RB, rs RB + RB) of a slice of 256 columns of one layer in registers (RB = 4 RPT rows), so each
// stored element is read from HBM once per product, in runs of 1 KB.
//   A. partial sums r_g[u] = sum_{j in slice} P[u][j] q[j]  ->  part[g][u]
//   B. the first `nfolders` work-groups fold, in a fixed order, 32-row chunks of the partial vectors of
//      all column slices of a row slice, add q^L (full mode), double (B = 2I), write rbar and t^L
//   C. every work-group reads the rbar of its rows and forms t[j] = sum_u P[u][j] rbar[u] from its registers;
//      with several row slices these are partial sums over u, written per row slice and added by
//      team_fold_t_kernel afterwards.
// The kernel is persistent: the host sizes the grid (teams x G) to be resident all at once, and team t
// walks over samples t, t + teams, ...
// Exchange between work-groups: every exchanged float travels in a 64-bit word together with a
// sequence number (seq_base + samples done + 1, never 0), written and read with single device-scope
// atomic accesses.  Those go through to memory, past the XCD-private L2s, so no cache write-back or
// invalidation is needed (measured: device-scope fences around plain accesses, which flush and
// invalidate a whole L2 each time, made this kernel 16x slower than the two-pass kernels), and a reader
// simply polls the word until it carries the expected number: no counters, no store-then-signal round
// trips.  Two sets of words are used alternately: a work-group writes set k & 1 for its k-th sample after
// it has read rbar of sample k-1, which exists only after every work-group of the team has written
// sample k-1 and so is done reading sample k-2, the previous user of that set.
// Every wait is bounded: after spin_limit polls a thread raises the error word and its work-group
// leaves; so does every work-group that sees the error word raised.  The host reports that as an error.
struct TeamArgs {
    StreamArgs a;
    int G;                               // work-groups per team = nrs * ncs
    int teams;
    int nrs;                             // row slices of RB rows
    int ncs;                             // column slices of 256 columns, all streamed layers together
    int slice_begin[DN_MAX_LAYERS + 1];  // first column slice of streamed layer m (1..L-2)
    int ntasks;                          // fold tasks per sample: (RB / 32) * nrs * (per-layer mode: L-2, else 1)
    int nfolders;                        // work-groups that fold: min(G, ntasks)
    unsigned seq_base;
    unsigned long long* part;            // [teams][2][G][RB]
    unsigned long long* rbar;            // [teams][2][L-2 or 1][nrs * RB]
    float* tpart[DN_MAX_LAYERS + 1];     // nrs > 1: per streamed layer, [nrs][s][ld_m] partial t
    unsigned* error;                     // one word, nonzero after a wait ran out
    unsigned spin_limit;
};

__device__ __forceinline__ unsigned long long ll_pack(float v, unsigned seq) {
    return ((unsigned long long)seq << 32) | (unsigned long long)__builtin_bit_cast(unsigned, v);
}
__device__ __forceinline__ void ll_store(unsigned long long* p, float v, unsigned seq) {
    __hip_atomic_store(p, ll_pack(v, seq), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ unsigned long long ll_load(const unsigned long long* p) {
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Sum of the floats in base[k * stride], k = lo, lo + step, ... < hi, in that order, each taken once its
// word carries `seq`.  B words are polled together.  Returns false if a wait ran out (error word raised).
template <int B>
__device__ __forceinline__ bool ll_sum(const unsigned long long* base, long long stride, int lo, int hi, int step,
                                       unsigned seq, unsigned* error, unsigned spin_limit, float& out) {
    float acc = 0.f;
    for (int k0 = lo; k0 < hi; k0 += B * step) {
        unsigned long long w[B];
        bool got = false;
        for (unsigned spins = 0; spins < spin_limit; ++spins) {
            bool all = true;
#pragma unroll
            for (int b = 0; b < B; ++b) {
                w[b] = (k0 + b * step < hi) ? ll_load(base + (long long)(k0 + b * step) * stride)
                                            : ((unsigned long long)seq << 32);
                all = all && ((unsigned)(w[b] >> 32) == seq);
            }
            if (all) { got = true; break; }
            if ((spins & 63u) == 63u && __hip_atomic_load(error, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0u) break;
            __builtin_amdgcn_s_sleep(4);
        }
        if (!got) {
            __hip_atomic_store(error, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            out = 0.f;
            return false;
        }
#pragma unroll
        for (int b = 0; b < B; ++b) acc += __builtin_bit_cast(float, (unsigned)(w[b] & 0xffffffffull));
    }
    out = acc;
    return true;
}

// RPT rows per thread; thread (lane = float4 column, wave = row group) owns rows u0 + wave + 4 k, k < RPT.
// The last RL of a thread's rows live in LDS instead of registers (each thread reads back only what it
// wrote): with RPT = 32 that brings the kernel under the register budget of three work-groups per CU.
template <int RPT, int RL, int WAVES_PER_SIMD>
__global__ __launch_bounds__(256, WAVES_PER_SIMD) void jv_jtv_team_kernel(const TeamArgs ta) {
    constexpr int RB = 4 * RPT;                // rows per work-group
    constexpr int CW = 256;                    // columns per work-group
    constexpr int RR = RPT - RL;               // rows per thread kept in registers
    __shared__ float4 plds[RL > 0 ? RL : 1][256];
    const StreamArgs& a = ta.a;
    __shared__ float rl[RB];                   // partial r of this slice, later rbar of its rows
    __shared__ float fold[8][32];
    __shared__ __attribute__((aligned(16))) float tred[4][CW];
    __shared__ int flag;

    const int team = blockIdx.x / ta.G, g = blockIdx.x - team * ta.G;
    const int rs = g / ta.ncs, cs = g - rs * ta.ncs;
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    // the wave index as a scalar: row addresses are then scalar bases plus one per-lane column offset
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    int m = 1;
    for (int mm = 2; mm + 1 < a.L; ++mm)
        if (cs >= ta.slice_begin[mm]) m = mm;
    const int j = (cs - ta.slice_begin[m]) * CW + 4 * lane;
    const bool live = j < a.n[m];
    const int rem = live ? a.n[m] - j : 0;
    const long long ldm = a.ld[m];
    const int nL = a.nL;
    const int u0 = rs * RB;
    const int nlay = a.blockdiag ? a.L - 2 : 1;
    const long long rows_all = (long long)ta.nrs * RB;
    unsigned long long* part_team = ta.part + (long long)team * 2 * ta.G * RB;
    unsigned long long* rbar_team = ta.rbar + (long long)team * 2 * nlay * rows_all;

    // a wait that ran out in an earlier launch: do nothing (the host reports the error word)
    if (tid == 0) flag = __hip_atomic_load(ta.error, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == 0u ? 1 : 0;
    __syncthreads();
    if (!flag) return;

    unsigned done = 0;        // samples this team has finished
    for (int i = team; i < a.s; i += ta.teams, ++done) {
        const unsigned seq = ta.seq_base + done + 1u;
        unsigned long long* part_cur = part_team + (long long)(done & 1u) * ta.G * RB;
        unsigned long long* rbar_cur = rbar_team + (long long)(done & 1u) * nlay * rows_all;
        // ---- A: load the slice, partial J v ------------------------------------------------
        float4 p[RR];
        float4 q4 = make_float4(0.f, 0.f, 0.f, 0.f);
        const float* __restrict__ prow = a.P[m] + ((long long)i * nL + u0 + wave) * ldm;    // uniform in the wave
        // columns past n_m are padding (never written): keep them out of the sums
        auto mask = [&](float4& x) {
            if (rem < 4) { x.w = 0.f; if (rem < 3) x.z = 0.f; if (rem < 2) x.y = 0.f; if (rem < 1) x.x = 0.f; }
        };
        auto row = [&](int k) {
            float4 x = make_float4(0.f, 0.f, 0.f, 0.f);
            if (live && u0 + wave + 4 * k < nL)
                x = *reinterpret_cast<const float4*>(prow + (long long)(4 * k) * ldm + j);
            return x;
        };
#pragma unroll
        for (int k = 0; k < RL; ++k) {                    // rows RR .. RPT-1 go to LDS
            float4 x = row(RR + k);
            mask(x);
            plds[k][tid] = x;
        }
#pragma unroll
        for (int k = 0; k < RR; ++k) p[k] = row(k);
        if (live) q4 = *reinterpret_cast<const float4*>(a.Q[m] + (long long)i * ldm + j);
        mask(q4);
#pragma unroll
        for (int k = 0; k < RR; ++k) mask(p[k]);
#pragma unroll
        for (int k = 0; k < RPT; ++k) {
            const float4 pk = k < RR ? p[k < RR ? k : 0] : plds[k < RR ? 0 : k - RR][tid];
            float x = pk.x * q4.x + pk.y * q4.y + pk.z * q4.z + pk.w * q4.w;
            x = wave_sum_to_lane63(x);
            if (lane == 63) rl[wave + 4 * k] = x;         // rows past n_L get zeros (p was zero)
        }
        __syncthreads();
        for (int u = tid; u < RB; u += 256) ll_store(&part_cur[(long long)g * RB + u], rl[u], seq);

        // ---- B: fold the partial vectors (first nfolders work-groups) -------------------------
        bool ok = true;
        if (g < ta.nfolders) {
            for (int task = g; task < ta.ntasks; task += ta.nfolders) {
                // task -> (layer, row slice, 32-row chunk)
                constexpr int CH = RB / 32;
                const int c = task % CH;
                const int trs = (task / CH) % ta.nrs;
                const int lay = a.blockdiag ? task / (CH * ta.nrs) + 1 : 0;     // 0: all layers together
                const int c_lo = a.blockdiag ? ta.slice_begin[lay] : 0;
                const int c_hi = a.blockdiag ? (lay + 2 < a.L ? ta.slice_begin[lay + 1] : ta.ncs) : ta.ncs;
                const int ul = tid & 31, sl = tid >> 5;
                float acc = 0.f;
                ok = ll_sum<8>(part_cur + ((long long)trs * ta.ncs) * RB + c * 32 + ul, RB, c_lo + sl, c_hi, 8, seq,
                               ta.error, ta.spin_limit, acc) && ok;
                __syncthreads();
                fold[sl][ul] = acc;
                __syncthreads();
                if (tid < 32) {
                    const int u = trs * RB + c * 32 + tid;
                    float r = ((fold[0][tid] + fold[1][tid]) + (fold[2][tid] + fold[3][tid])) +
                              ((fold[4][tid] + fold[5][tid]) + (fold[6][tid] + fold[7][tid]));
                    if (u < nL) {
                        const float qL = a.Q[a.L][(long long)i * a.ld[a.L] + u];
                        if (!a.blockdiag) {
                            r = 2.0f * (r + qL);
                            a.T[a.L][(long long)i * a.ld[a.L] + u] = r;
                        } else {
                            r = 2.0f * r;
                            if (lay == 1) a.T[a.L][(long long)i * a.ld[a.L] + u] = 2.0f * qL;
                        }
                    }
                    ll_store(&rbar_cur[(long long)(a.blockdiag ? lay - 1 : 0) * rows_all + u], r, seq);
                }
            }
        }

        // ---- C: transposed product from the registers ------------------------------------------
        {
            const unsigned long long* my_rbar = rbar_cur + (long long)(a.blockdiag ? m - 1 : 0) * rows_all + u0;
            for (int u = tid; u < RB; u += 256) {
                float v = 0.f;
                ok = ll_sum<1>(my_rbar + u, 0, 0, 1, 1, seq, ta.error, ta.spin_limit, v) && ok;
                rl[u] = v;
            }
        }
        if (!__syncthreads_and(ok ? 1 : 0)) return;
        float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
        for (int k = 0; k < RPT; ++k) {
            const float w = rl[wave + 4 * k];             // zero for rows past n_L
            const float4 pk = k < RR ? p[k < RR ? k : 0] : plds[k < RR ? 0 : k - RR][tid];
            acc.x += pk.x * w; acc.y += pk.y * w; acc.z += pk.z * w; acc.w += pk.w * w;
        }
        *reinterpret_cast<float4*>(&tred[wave][4 * lane]) = acc;
        __syncthreads();
        if (tid < 64 && live) {
            float4 t0 = *reinterpret_cast<const float4*>(&tred[0][4 * lane]);
            const float4 t1 = *reinterpret_cast<const float4*>(&tred[1][4 * lane]);
            const float4 t2 = *reinterpret_cast<const float4*>(&tred[2][4 * lane]);
            const float4 t3 = *reinterpret_cast<const float4*>(&tred[3][4 * lane]);
            t0.x = (t0.x + t1.x) + (t2.x + t3.x); t0.y = (t0.y + t1.y) + (t2.y + t3.y);
            t0.z = (t0.z + t1.z) + (t2.z + t3.z); t0.w = (t0.w + t1.w) + (t2.w + t3.w);
            float* dst = ta.nrs > 1 ? ta.tpart[m] + ((long long)rs * a.s + i) * ldm + j
                                    : a.T[m] + (long long)i * ldm + j;
            *reinterpret_cast<float4*>(dst) = t0;
        }
        __syncthreads();      // rl, fold and tred are reused by the next sample
    }
}

// exchange words to zero (sequence number 0 = nothing written) once after the workspace is bound
__global__ void team_clear_kernel(unsigned long long* words, long long n, unsigned* error) {
    for (long long e = (long long)blockIdx.x * blockDim.x + threadIdx.x; e < n; e += (long long)gridDim.x * blockDim.x)
        words[e] = 0ull;
    if (blockIdx.x == 0 && threadIdx.x == 0) *error = 0u;
}

// t^{m,i} = sum over the row slices of the partial transposed products (fixed order)
__global__ __launch_bounds__(256) void team_fold_t_kernel(const float* __restrict__ tpart, float* __restrict__ T,
                                                          int nrs, long long total4) {
    const long long slab4 = total4;   // float4 per row slice
    for (long long e = (long long)blockIdx.x * 256 + threadIdx.x; e < total4; e += (long long)gridDim.x * 256) {
        float4 acc = reinterpret_cast<const float4*>(tpart)[e];
        for (int r = 1; r < nrs; ++r) {
            const float4 x = reinterpret_cast<const float4*>(tpart)[(long long)r * slab4 + e];
            acc.x += x.x; acc.y += x.y; acc.z += x.z; acc.w += x.w;
        }
        reinterpret_cast<float4*>(T)[e] = acc;
    }
}

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
    int blk_begin[DN_MAX_LAYERS + 2];   // first work-group of layer m; one work-group = (row j, 1024 columns)
    int chunks[DN_MAX_LAYERS + 1];      // 1024-column chunks per row of layer m
};

typedef float f32x4v __attribute__((ext_vector_type(4), aligned(4)));

__global__ __launch_bounds__(256) void tn_reduce_kernel(const ReduceArgs a, const float* __restrict__ x,
                                                        float* __restrict__ out, float invC, float scale) {
    int m = 1;
#pragma unroll
    for (int k = 2; k <= DN_MAX_LAYERS; ++k)
        if (k <= a.L && (int)blockIdx.x >= a.blk_begin[k]) m = k;
    const int loc = (int)blockIdx.x - a.blk_begin[m];
    const int j = loc / a.chunks[m];
    const int t = (loc - j * a.chunks[m]) * 1024 + 4 * (int)threadIdx.x;
    const int np = a.n[m - 1];
    if (t > np) return;                       // columns 0..np (np = bias column)
    const float* __restrict__ w = a.W[m] + (long long)j * a.ldw[m] + t;   // 16-byte aligned: ldw % 4 == 0
    const long long ss = a.split_stride[m];
    const int ns = a.splits[m];
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
        o[0] = xv[0] * invC + scale * s4[0];
        o[1] = xv[1] * invC + scale * s4[1];
        o[2] = xv[2] * invC + scale * s4[2];
        o[3] = xv[3] * invC + scale * s4[3];
        *reinterpret_cast<f32x4v*>(out + wbase + t) = o;
    } else {
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const int tt = t + c;
            if (tt < np)       out[wbase + tt] = x[wbase + tt] * invC + scale * s4[c];
            else if (tt == np) out[bidx] = x[bidx] * invC + scale * s4[c];
        }
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

// partial p^T (q + lambda p)
__global__ __launch_bounds__(256) void cg_dot_kernel(const CgSegs sg, const float* __restrict__ p,
                                                     const float* __restrict__ q, float lambda,
                                                     double* __restrict__ partials) {
    __shared__ double red[4];
    int seg; long long lo, hi;
    cg_locate(sg, seg, lo, hi);
    double acc = 0.0;
    cg_sweep(lo, hi,
             [&](long long e) {
                 const f32x4v pe = ld4(p + e), qe = ld4(q + e);
                 double s4[4];
#pragma unroll
                 for (int k = 0; k < 4; ++k) s4[k] = (double)pe[k] * (double)(qe[k] + lambda * pe[k]);
                 acc += (s4[0] + s4[1]) + (s4[2] + s4[3]);
             },
             [&](long long e) {
                 const float pe = p[e];
                 acc += (double)pe * (double)(q[e] + lambda * pe);
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
    const double pq = block_sum_range(pq_partials, sg.cb[seg], sg.cb[seg + 1], red);
    const float alpha = (float)(st->rho[seg] / pq);
    double acc = 0.0;
    cg_sweep(lo, hi,
             [&](long long e) {
                 const f32x4v pe = ld4(p + e), qe = ld4(q + e);
                 f32x4v de = ld4(d + e), re = ld4(r + e);
                 double s4[4];
#pragma unroll
                 for (int k = 0; k < 4; ++k) {
                     de[k] += alpha * pe[k];
                     re[k] = re[k] - alpha * (qe[k] + lambda * pe[k]);
                     s4[k] = (double)re[k] * (double)re[k];
                 }
                 st4(d + e, de); st4(r + e, re);
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

// rho' = r^T r;  stop test ||r|| <= sigma ||g||;  beta = rho'/rho;  p = r + beta p
__global__ __launch_bounds__(256) void cg_update_p_kernel(const CgSegs sg, const CgState* __restrict__ st_cur,
                                                          CgState* __restrict__ st_next,
                                                          const double* __restrict__ rr_partials, double sigma2,
                                                          const float* __restrict__ r, float* __restrict__ p) {
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
             },
             [&](long long e) { p[e] = r[e] + beta * p[e]; });
}

// ---------------------------------------------------------------------------------------------
// Block-diagonal product for a general split structure (variable partitions of Section 3.1; Section 4.1).
// Layer m has ga = split[m-1] input groups and gb = split[m] output groups; partition (a, b) owns the weights
// from input group a to output group b (and, for a = 0, the biases of group b).  For each input group a the
// inner sums over t in that group are Q^{m,a} (one dense product each); per partition
//   r^{(a,b)}_i[u] = sum_{j in group b} P^m_i[u][j] q^{m,a,i}_j,     t^{m,a,i}_j = sum_u P^m_i[u][j] 2 r^{(a,b(j))}_i[u].
// jv_part_kernel / jtv_part_kernel are the general (two-pass) form, jv_jtv_fused_part_kernel the single-pass
// one for small outputs; all hidden layers' blocks are streamed.
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
    // single-pass kernel: strip slot k is 256 columns of layer wlayer[k], starting at 256 * wcol[k]
    int nwslots;
    int wlayer[DN_MAX_WSLOTS];
    int wcol[DN_MAX_WSLOTS];
};

__device__ __forceinline__ int group_of(const int* bound, int groups, int j) {
    int g = 0;
#pragma unroll
    for (int k = 1; k < DN_MAX_SPLIT; ++k)
        if (k < groups && j >= bound[k]) g = k;
    return g;
}

// work-group = (sample, block of 4 outputs); each wave takes one row u of every hidden layer's block
__global__ __launch_bounds__(256) void jv_part_kernel(const PartArgs a) {
    constexpr int UB = 4;
    const int ublocks = (a.nL + UB - 1) / UB;
    const int i = blockIdx.x / ublocks;
    const int u0 = (blockIdx.x - i * ublocks) * UB;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const long long slab = (long long)a.s * a.ldr;
    for (int uu = wave; uu < UB; uu += 4) {
        const int u = u0 + uu;
        if (u >= a.nL) break;
        for (int m = 1; m < a.L; ++m) {
            const int ga = a.split[m - 1], gb = a.split[m];
            const float* __restrict__ prow = a.P[m] + ((long long)i * a.nL + u) * a.ld[m];
            double acc[DN_MAX_SPLIT][DN_MAX_SPLIT];
#pragma unroll
            for (int x = 0; x < DN_MAX_SPLIT; ++x)
#pragma unroll
                for (int y = 0; y < DN_MAX_SPLIT; ++y) acc[x][y] = 0.0;
            // four columns at a time (rows are 16-byte aligned and padded to a multiple of 4 floats; the padding of
            // P and Q holds no data, so the last, partial group of four is masked); a group boundary may fall
            // inside a group of four, hence the per-column group index
            const int nm4 = (a.n[m] + 3) >> 2;
            for (int c4 = lane; c4 < nm4; c4 += 64) {
                const int j = 4 * c4;
                const float4 p4 = *reinterpret_cast<const float4*>(prow + j);
                const float pe[4] = {p4.x, p4.y, p4.z, p4.w};
                int bj[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) bj[e] = (j + e < a.n[m]) ? group_of(a.bound[m], gb, j + e) : -1;
#pragma unroll
                for (int x = 0; x < DN_MAX_SPLIT; ++x) {
                    if (x < ga) {
                        const float4 q4 = *reinterpret_cast<const float4*>(a.Qp[m] + ((long long)x * a.s + i) * a.ld[m] + j);
                        const float qe[4] = {q4.x, q4.y, q4.z, q4.w};
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            const double t = bj[e] >= 0 ? (double)pe[e] * (double)qe[e] : 0.0;
#pragma unroll
                            for (int y = 0; y < DN_MAX_SPLIT; ++y) acc[x][y] += (y == bj[e]) ? t : 0.0;
                        }
                    }
                }
            }
#pragma unroll
            for (int x = 0; x < DN_MAX_SPLIT; ++x)
#pragma unroll
                for (int y = 0; y < DN_MAX_SPLIT; ++y) {
                    if (x < ga && y < gb) {
                        const double t = wave_sum_d(acc[x][y]);
                        if (lane == 0)
                            a.R[(long long)(a.part_base[m] + x * gb + y) * slab + (long long)i * a.ldr + u] = (float)t;
                    }
                }
        }
    }
}

// work-group = (sample, layer, chunk of 256 columns); one thread per column.  Layer L: t^{L,a} = 2 q^{L,a}.
__global__ __launch_bounds__(256) void jtv_part_kernel(const PartArgs a, int chunks_total) {
    extern __shared__ float rbar[];          // [ga][gb][nL] of this layer
    const int i = blockIdx.x / chunks_total;
    int c = blockIdx.x - i * chunks_total;
    int m = 1;
    for (; m < a.L; ++m) {
        const int cm = (a.n[m] + 255) >> 8;
        if (c < cm) break;
        c -= cm;
    }
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
    const int j = (c << 8) + threadIdx.x;
    if (j >= a.n[m]) return;
    const int bj = group_of(a.bound[m], gb, j);
    const float* __restrict__ pcol = a.P[m] + (long long)i * a.nL * a.ld[m] + j;
    double acc[DN_MAX_SPLIT];
#pragma unroll
    for (int x = 0; x < DN_MAX_SPLIT; ++x) acc[x] = 0.0;
#pragma unroll 4
    for (int u = 0; u < a.nL; ++u) {
        const double pj = (double)pcol[(long long)u * a.ld[m]];
#pragma unroll
        for (int x = 0; x < DN_MAX_SPLIT; ++x)
            if (x < ga) acc[x] += pj * (double)rbar[(x * gb + bj) * a.nL + u];
    }
#pragma unroll
    for (int x = 0; x < DN_MAX_SPLIT; ++x)
        if (x < ga) a.Tp[m][((long long)x * a.s + i) * a.ld[m] + j] = (float)acc[x];
}

// Both passes in one for a split structure when n_L <= NLMAX and the hidden widths fit one work-group: the
// strips of P^m_i stay in registers as in jv_jtv_fused_kernel; per input group x the partial sums are kept
// apart by the output group of each column, and the transposed product picks, column by column, the r of
// that column's partition.  One HBM read of the stored blocks per product.
template <int NLMAX, int CH>
__global__ __launch_bounds__(1024) void jv_jtv_fused_part_kernel(const PartArgs a) {
    __shared__ float part[DN_MAX_WSLOTS][DN_MAX_SPLIT][NLMAX];          // [slot][output group][u], one x at a time
    __shared__ float rb[DN_MAX_LAYERS][DN_MAX_SPLIT][NLMAX];            // [layer][output group][u], one x at a time
    const int i = blockIdx.x;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int nwaves = blockDim.x >> 6;
    int m[CH], j[CH], bj[CH][4], ylo[CH], yhi[CH];
    bool live[CH];
    float4 p[CH][NLMAX];
    int gamax = 1;
    for (int mm = 1; mm < a.L; ++mm) gamax = max(gamax, a.split[mm - 1]);
#pragma unroll
    for (int ch = 0; ch < CH; ++ch) {
        const int slot = wave + ch * nwaves;
        const bool have = slot < a.nwslots;
        m[ch] = have ? a.wlayer[slot] : 1;
        j[ch] = have ? 4 * (64 * a.wcol[slot] + lane) : 0;
        live[ch] = have && j[ch] < a.n[m[ch]];
        {
            // output groups of the first and last column of this strip slot (same for all lanes)
            const int c0 = have ? 256 * a.wcol[slot] : 0;
            ylo[ch] = group_of(a.bound[m[ch]], a.split[m[ch]], c0);
            yhi[ch] = group_of(a.bound[m[ch]], a.split[m[ch]], min(c0 + 255, a.n[m[ch]] - 1));
        }
        const long long ldm = a.ld[m[ch]];
        const float* __restrict__ pbase = a.P[m[ch]] + (long long)i * a.nL * ldm + j[ch];
#pragma unroll
        for (int u = 0; u < NLMAX; ++u) {
            p[ch][u] = make_float4(0.f, 0.f, 0.f, 0.f);
            if (live[ch] && u < a.nL) p[ch][u] = *reinterpret_cast<const float4*>(pbase + (long long)u * ldm);
        }
        // output group of each of the four columns; -1 for padding columns (and their P values cleared)
        const int rem = live[ch] ? a.n[m[ch]] - j[ch] : 0;
#pragma unroll
        for (int e = 0; e < 4; ++e) bj[ch][e] = e < rem ? group_of(a.bound[m[ch]], a.split[m[ch]], j[ch] + e) : -1;
        if (rem < 4) {
#pragma unroll
            for (int u = 0; u < NLMAX; ++u) {
                p[ch][u].w = 0.f; if (rem < 3) p[ch][u].z = 0.f; if (rem < 2) p[ch][u].y = 0.f; if (rem < 1) p[ch][u].x = 0.f;
            }
        }
    }
    // output layer (identity block): t^{L,x} = 2 q^{L,x}
    for (int x = 0; x < a.split[a.L - 1]; ++x)
        for (int u = threadIdx.x; u < a.nL; u += blockDim.x) {
            const long long e = ((long long)x * a.s + i) * a.ld[a.L] + u;
            a.Tp[a.L][e] = 2.0f * a.Qp[a.L][e];
        }
    for (int x = 0; x < gamax; ++x) {
        // ---- partial sums of this input group, kept apart by output group -------------------------
#pragma unroll
        for (int ch = 0; ch < CH; ++ch) {
            const int slot = wave + ch * nwaves;
            const bool on = live[ch] && x < a.split[m[ch] - 1];
            float4 q4 = make_float4(0.f, 0.f, 0.f, 0.f);
            if (on) q4 = *reinterpret_cast<const float4*>(a.Qp[m[ch]] + ((long long)x * a.s + i) * a.ld[m[ch]] + j[ch]);
            // padding columns of Q are never written
            if (bj[ch][0] < 0) q4.x = 0.f;
            if (bj[ch][1] < 0) q4.y = 0.f;
            if (bj[ch][2] < 0) q4.z = 0.f;
            if (bj[ch][3] < 0) q4.w = 0.f;
#pragma unroll
            for (int u = 0; u < NLMAX; ++u) {
                if (u < a.nL) {
                    const float t0 = p[ch][u].x * q4.x, t1 = p[ch][u].y * q4.y, t2 = p[ch][u].z * q4.z,
                                t3 = p[ch][u].w * q4.w;
#pragma unroll
                    for (int y = 0; y < DN_MAX_SPLIT; ++y) {
                        // only the output groups that this strip's 256 columns touch need a reduction (uniform
                        // in the wave); the others get a plain zero
                        float v = 0.f;
                        if (y >= ylo[ch] && y <= yhi[ch]) {
                            v = (bj[ch][0] == y ? t0 : 0.f) + (bj[ch][1] == y ? t1 : 0.f) +
                                (bj[ch][2] == y ? t2 : 0.f) + (bj[ch][3] == y ? t3 : 0.f);
                            v = wave_sum_to_lane63(v);
                        }
                        if (lane == 63 && slot < a.nwslots) part[slot][y][u] = v;
                    }
                }
            }
        }
        __syncthreads();
        // ---- r of every partition (layer, x, y), doubled: B = 2I ----------------------------------
        for (int e = threadIdx.x; e < (a.L - 1) * DN_MAX_SPLIT * NLMAX; e += blockDim.x) {
            const int u = e % NLMAX, y = (e / NLMAX) % DN_MAX_SPLIT, mm = e / (NLMAX * DN_MAX_SPLIT) + 1;
            float rsum = 0.f;
            for (int w = 0; w < a.nwslots; ++w)
                if (a.wlayer[w] == mm) rsum += part[w][y][u];
            rb[mm][y][u] = 2.0f * rsum;
        }
        __syncthreads();
        // ---- transposed product: column j takes the r of its own partition -------------------------
#pragma unroll
        for (int ch = 0; ch < CH; ++ch) {
            if (live[ch] && x < a.split[m[ch] - 1]) {
                float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
                const int y0 = bj[ch][0];
#pragma unroll
                for (int u = 0; u < NLMAX; ++u) {
                    if (u < a.nL) {
                        const float w0 = rb[m[ch]][y0][u];
                        const float w1 = bj[ch][1] == y0 ? w0 : (bj[ch][1] >= 0 ? rb[m[ch]][bj[ch][1]][u] : 0.f);
                        const float w2 = bj[ch][2] == y0 ? w0 : (bj[ch][2] >= 0 ? rb[m[ch]][bj[ch][2]][u] : 0.f);
                        const float w3 = bj[ch][3] == y0 ? w0 : (bj[ch][3] >= 0 ? rb[m[ch]][bj[ch][3]][u] : 0.f);
                        acc.x += p[ch][u].x * w0; acc.y += p[ch][u].y * w1; acc.z += p[ch][u].z * w2; acc.w += p[ch][u].w * w3;
                    }
                }
                *reinterpret_cast<float4*>(a.Tp[m[ch]] + ((long long)x * a.s + i) * a.ld[m[ch]] + j[ch]) = acc;
            }
        }
        // part and rb are rewritten for the next input group only after the barrier at the top of its second
        // stage has been passed by everyone, i.e. after all reads above have been issued and completed
        __syncthreads();
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
    if (j < a.n[m])
        for (int i = i_lo + r; i < i_hi; i += 16) acc += (double)a.T0[m][(long long)i * a.ld[m] + j];
    red[r][c] = acc;
    __syncthreads();
    if (r == 0 && j < a.n[m]) {
        double t = 0.0;
#pragma unroll
        for (int k = 0; k < 16; ++k) t += red[k][c];
        a.W[m][(long long)sidx * a.n[m] * a.ldw[m] + (long long)j * a.ldw[m] + a.n[m - 1]] = (float)t;
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
