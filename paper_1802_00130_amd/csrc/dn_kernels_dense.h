// Small dense-side kernels: row gather, first stored block, padded copies and transposes, the loss and
// the objective value.
#pragma once
#include "dn_common.h"

namespace dn {

// ---------------------------------------------------------------------------------------------
// Row gather: XS[i][:] = X[S[i]][:]   (the subsample of Section 4.3)
__global__ __launch_bounds__(256) void gather_rows_kernel(const float* __restrict__ X, const int* __restrict__ S,
                                                          float* __restrict__ XS, int s, int n0, int l,
                                                          long long ldx, long long ldxs) {
    // one wave per row at a time: 4 rows per work-group and pass
    const int lane = threadIdx.x & 63;
    for (int i = blockIdx.x * 4 + (threadIdx.x >> 6); i < s; i += gridDim.x * 4) {
        const int row = min(max(S[i], 0), l - 1);  // ids outside [0, l) are clamped, never dereferenced
        const float* __restrict__ src = X + (long long)row * ldx;
        float* __restrict__ dst = XS + (long long)i * ldxs;
        // 16-byte accesses that only assume the alignment of a float (rows of X start anywhere)
        typedef float f4u __attribute__((ext_vector_type(4), aligned(4)));
        const int n4 = n0 & ~3;
        for (int t = 4 * lane; t < n4; t += 256) *reinterpret_cast<f4u*>(dst + t) = *reinterpret_cast<const f4u*>(src + t);
        if (n4 + lane < n0) dst[n4 + lane] = src[n4 + lane];
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

// dst[c][r] = src[r][c] for c < cols, and one more row dst[cols][r] = 1: the activations of the subsample with the
// sample index contiguous and the constant input of the bias terms as a last row (Section 4.2: the outer sums over
// samples then read this operand K-contiguously; it is the same for every product until the next dn_jacobian_prep).
__global__ __launch_bounds__(256) void transpose_ones_kernel(const float* __restrict__ src, long long lds_src,
                                                             float* __restrict__ dst, long long ld_dst, int rows,
                                                             int cols) {
    __shared__ float tile[32][33];
    const int bx = blockIdx.x * 32, by = blockIdx.y * 32;
    const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;   // 32 x 8
#pragma unroll
    for (int k = 0; k < 32; k += 8) {
        const int rr = by + ty + k, cc = bx + tx;
        if (rr < rows && cc < cols) tile[ty + k][tx] = src[(long long)rr * lds_src + cc];
    }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < 32; k += 8) {
        const int cc = bx + ty + k, rr = by + tx;
        if (rr < rows && cc < cols) dst[(long long)cc * ld_dst + rr] = tile[tx][ty + k];
    }
    if (blockIdx.x == 0) {
        const int rr = by + (threadIdx.x & 31);
        if (threadIdx.x < 32 && rr < rows) dst[(long long)cols * ld_dst + rr] = 1.0f;
    }
}

// dst_p[c][r] = src_p[r][c] for up to DN_MAX_LAYERS matrices of `rows` rows in one launch (64 x 64 tiles, 16-byte
// accesses on both sides): the left operands T^m of the outer sums over samples (Section 4.2) with the sample index
// contiguous, for the launches large enough that a K-contiguous operand pays for the copy.  Rows of dst are ld_dst
// floats (a multiple of 4, >= rows rounded up to 4); the padding columns are written as zeros.
struct TransposeArgs {
    int nprob, rows, tiles_r;
    const float* src[DN_MAX_LAYERS];
    float* dst[DN_MAX_LAYERS];
    long long ld_src[DN_MAX_LAYERS];
    int cols[DN_MAX_LAYERS];
    int first[DN_MAX_LAYERS + 1];     // first work-group of each matrix
    long long ld_dst;
};

__global__ __launch_bounds__(256) void transpose_group_kernel(const TransposeArgs a) {
    __shared__ float tile[64][65];
    int p = 0;
#pragma unroll
    for (int i = 1; i < DN_MAX_LAYERS; ++i)
        if (i < a.nprob && (int)blockIdx.x >= a.first[i]) p = i;
    const int b = blockIdx.x - a.first[p];
    const int r0 = (b % a.tiles_r) * 64, c0 = (b / a.tiles_r) * 64;
    const int cols = a.cols[p];
    const float* __restrict__ src = a.src[p];
    float* __restrict__ dst = a.dst[p];
    const long long lds = a.ld_src[p];
    const int q = threadIdx.x & 15, w = threadIdx.x >> 4;      // 16 quads of columns x 16 rows per pass
#pragma unroll
    for (int k = 0; k < 64; k += 16) {
        const int rr = r0 + w + k, cc = c0 + 4 * q;
        float4 x = make_float4(0.f, 0.f, 0.f, 0.f);
        if (rr < a.rows) {
            const float* s4 = src + (long long)rr * lds + cc;
            if (cc + 3 < cols) {
                x = *reinterpret_cast<const float4*>(s4);
            } else {
                if (cc + 0 < cols) x.x = s4[0];
                if (cc + 1 < cols) x.y = s4[1];
                if (cc + 2 < cols) x.z = s4[2];
            }
        }
        tile[w + k][4 * q + 0] = x.x; tile[w + k][4 * q + 1] = x.y;
        tile[w + k][4 * q + 2] = x.z; tile[w + k][4 * q + 3] = x.w;
    }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < 64; k += 16) {
        const int cc = c0 + w + k, rr = r0 + 4 * q;          // a row of dst, four consecutive samples
        if (cc < cols && rr < a.rows)
            *reinterpret_cast<float4*>(dst + (long long)cc * a.ld_dst + rr) =
                make_float4(tile[4 * q + 0][w + k], tile[4 * q + 1][w + k], tile[4 * q + 2][w + k], tile[4 * q + 3][w + k]);
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

}  // namespace dn
