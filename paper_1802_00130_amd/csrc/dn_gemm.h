// fp32 MFMA GEMM tile engine for gfx950 (CDNA4), 64-wide wavefronts.
//
// One kernel template serves every dense contraction of the path:
//   forward pass          Z^m = sigma(Z^{m-1} (W^m) + b^m)              (Section 2.1 forward recursion)
//   back-propagation      Delta^{m-1} = (Delta^m (W^m)^T) * sigma'      (Section 2.2)
//   Jacobian sweeps       P^{m-1} = (P^m (W^m)^T) * sigma'              (Section 3.3 recursion)
//   product inner sums    Q^m = Z^{m-1} V^m + vb^m                      (Section 4.2, sum over t)
//   sums over samples     T^m^T Z^{m-1}                                 (Section 2.2 / 4.2, sum over i)
//
// C[M x N] = op(A) op(B) with each operand stored either K-contiguous ("KC": [rows][K]) or
// row-contiguous ("RC": [K][rows]).  A launch covers up to DN_MAX_GROUP independent problems
// (one per layer) and optional split-K slices; blockIdx.x is a flat tile id.
//
// The MFMA used is v_mfma_f32_32x32x2_f32: per wave a 32x32 fp32 block accumulates two k
// values per instruction; lane (r = lane%32, h = lane/32) supplies A[r][k_h] and B[k_h][r] and
// holds C[8*(i/4) + 4*h + i%4][r] in accumulator register i (0..15).
// The k values handled by the two lane halves are any fixed pairing as long as A and B agree;
// here within each group of 8 consecutive k the half h takes k = 4h + j for step j = 0..3,
// which lets a K-contiguous operand be fetched from LDS with one 128-bit read per 4 MFMAs.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#define DN_MAX_GROUP 8

namespace dn {

typedef float f32x16 __attribute__((ext_vector_type(16)));

enum OperandLayout { KC = 0, RC = 1 };

enum Epilogue {
    EP_STORE = 0,         // C = acc
    EP_BIAS = 1,          // C = acc + bias[n]
    EP_BIAS_SIGMOID = 2,  // C = 1/(1+exp(-(acc + bias[n])))
    EP_DSIGMOID = 3       // C = acc * z(1-z), z = aux[(m / auxdiv) * ldaux + n]
};

struct GemmProblem {
    const float* A;
    const float* B;
    float* C;
    const float* bias;   // EP_BIAS*: length N
    const float* aux;    // EP_DSIGMOID: activations z
    long long lda, ldb, ldc, ldaux;
    long long split_stride;  // elements between the C outputs of consecutive K-slices
    int M, N, K;
    int auxdiv;          // aux row = output row / auxdiv
    int tiles_m, tiles_n;
    int splits;          // number of K-slices (>= 1)
    int k_per_split;     // multiple of the K tile
    int tile_begin;      // first flat tile id of this problem
    int a_vec, b_vec;    // 1 if 16-byte vector loads are legal for the operand
    int b_ones_col;      // 1: column N-1 of op(B) is a virtual column of ones (not read from memory)
};

struct GemmGroup {
    int nprob;
    int total_tiles;
    GemmProblem p[DN_MAX_GROUP];
};

__device__ __forceinline__ float sigmoidf_fast(float s) { return 1.0f / (1.0f + __expf(-s)); }

// ---- global -> register tile fetch -------------------------------------------------------
// A tile of an operand is ROWS x BK values.  KC: slot = (row, 4 consecutive k).
// RC: slot = (k, 4 consecutive rows).  Out-of-range elements are zero.
template <int ROWS, int BK, int LAYOUT, int NT>
struct TileFetch {
    static constexpr int SLOTS = ROWS * BK / 4;
    static constexpr int PER_THREAD = (SLOTS + NT - 1) / NT;
    float4 v[PER_THREAD];

    __device__ __forceinline__ void load(const float* __restrict__ base, long long ld, int row0, int k0,
                                         int rows_total, int k_end, int vec_ok, int ones_row, int tid) {
#pragma unroll
        for (int i = 0; i < PER_THREAD; ++i) {
            int s = tid + i * NT;
            float4 x = make_float4(0.f, 0.f, 0.f, 0.f);
            if (SLOTS % NT == 0 || s < SLOTS) {
                if (LAYOUT == KC) {
                    int row = row0 + s / (BK / 4);
                    int k = k0 + 4 * (s % (BK / 4));
                    if (row < rows_total) {
                        if (row == ones_row) {
                            x.x = (k + 0 < k_end) ? 1.f : 0.f;
                            x.y = (k + 1 < k_end) ? 1.f : 0.f;
                            x.z = (k + 2 < k_end) ? 1.f : 0.f;
                            x.w = (k + 3 < k_end) ? 1.f : 0.f;
                        } else {
                            const float* p = base + (long long)row * ld + k;
                            if (vec_ok && k + 3 < k_end) {
                                x = *reinterpret_cast<const float4*>(p);
                            } else {
                                if (k + 0 < k_end) x.x = p[0];
                                if (k + 1 < k_end) x.y = p[1];
                                if (k + 2 < k_end) x.z = p[2];
                                if (k + 3 < k_end) x.w = p[3];
                            }
                        }
                    }
                } else {
                    int k = k0 + s / (ROWS / 4);
                    int row = row0 + 4 * (s % (ROWS / 4));
                    if (k < k_end) {
                        const float* p = base + (long long)k * ld + row;
                        if (vec_ok && row + 3 < rows_total && (ones_row < row || ones_row > row + 3)) {
                            x = *reinterpret_cast<const float4*>(p);
                        } else {
                            if (row + 0 < rows_total) x.x = (row + 0 == ones_row) ? 1.f : p[0];
                            if (row + 1 < rows_total) x.y = (row + 1 == ones_row) ? 1.f : p[1];
                            if (row + 2 < rows_total) x.z = (row + 2 == ones_row) ? 1.f : p[2];
                            if (row + 3 < rows_total) x.w = (row + 3 == ones_row) ? 1.f : p[3];
                        }
                    }
                }
            }
            v[i] = x;
        }
    }

    // LDS strides: KC rows are BK+4 floats apart, RC k-rows are ROWS+8 floats apart.
    static constexpr int LDS_STRIDE = (LAYOUT == KC) ? (BK + 4) : (ROWS + 8);
    static constexpr int LDS_FLOATS = (LAYOUT == KC) ? ROWS * (BK + 4) : BK * (ROWS + 8);

    __device__ __forceinline__ void store(float* lds, int tid) const {
#pragma unroll
        for (int i = 0; i < PER_THREAD; ++i) {
            int s = tid + i * NT;
            if (SLOTS % NT == 0 || s < SLOTS) {
                int off;
                if (LAYOUT == KC) off = (s / (BK / 4)) * LDS_STRIDE + 4 * (s % (BK / 4));
                else              off = (s / (ROWS / 4)) * LDS_STRIDE + 4 * (s % (ROWS / 4));
                *reinterpret_cast<float4*>(lds + off) = v[i];
            }
        }
    }
};

// Fetch the four k-step values of one 32-row MFMA operand block for k-group kk (8 k values).
template <int ROWS, int BK, int LAYOUT>
__device__ __forceinline__ void frag_read(const float* lds, int row, int kk, int h, float (&f)[4]) {
    if (LAYOUT == KC) {
        float4 x = *reinterpret_cast<const float4*>(lds + row * (BK + 4) + kk * 8 + 4 * h);
        f[0] = x.x; f[1] = x.y; f[2] = x.z; f[3] = x.w;
    } else {
        const float* p = lds + (kk * 8 + 4 * h) * (ROWS + 8) + row;
        f[0] = p[0];
        f[1] = p[ROWS + 8];
        f[2] = p[2 * (ROWS + 8)];
        f[3] = p[3 * (ROWS + 8)];
    }
}

// BM x BN macro tile, 4 waves arranged WGM x WGN, each wave owning (BM/WGM) x (BN/WGN).
template <int BM, int BN, int BK, int WGM, int WGN, int LA, int LB, int EP>
__global__ __launch_bounds__(256) void gemm_kernel(const GemmGroup g) {
    constexpr int NT = 256;
    static_assert(WGM * WGN == 4, "four waves per work-group");
    constexpr int WM = BM / WGM, WN = BN / WGN;
    constexpr int FM = WM / 32, FN = WN / 32;
    static_assert(WM % 32 == 0 && WN % 32 == 0 && BK % 8 == 0, "tile shape");
    using FetchA = TileFetch<BM, BK, LA, NT>;
    using FetchB = TileFetch<BN, BK, LB, NT>;

    __shared__ __attribute__((aligned(16))) float ldsA[2][FetchA::LDS_FLOATS];
    __shared__ __attribute__((aligned(16))) float ldsB[2][FetchB::LDS_FLOATS];

    // ---- which problem / tile / K-slice ----
    const int bid = blockIdx.x;
    int pi = 0;
#pragma unroll
    for (int i = 1; i < DN_MAX_GROUP; ++i)
        if (i < g.nprob && bid >= g.p[i].tile_begin) pi = i;
    const GemmProblem& P = g.p[pi];
    int t = bid - P.tile_begin;
    const int tiles_mn = P.tiles_m * P.tiles_n;
    const int split = t / tiles_mn;
    t -= split * tiles_mn;
    // consecutive tile ids walk down M first so neighbouring work-groups share the B panel
    const int tm = t % P.tiles_m;
    const int tn = t / P.tiles_m;
    const int m0 = tm * BM, n0 = tn * BN;
    const int k_begin = split * P.k_per_split;
    const int k_end = min(P.K, k_begin + P.k_per_split);

    const int tid = threadIdx.x;
    const int wave = tid >> 6, lane = tid & 63;
    const int r = lane & 31, h = lane >> 5;
    const int wm0 = (wave / WGN) * WM, wn0 = (wave % WGN) * WN;

    const float* __restrict__ Ab = P.A;
    const float* __restrict__ Bb = P.B;
    const int ones_row = P.b_ones_col ? (P.N - 1) : -1;

    f32x16 acc[FM][FN];
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

    FetchA fa;
    FetchB fb;
    const int nk = (k_end - k_begin + BK - 1) / BK;
    if (nk > 0) {
        fa.load(Ab, P.lda, m0, k_begin, P.M, k_end, P.a_vec, -1, tid);
        fb.load(Bb, P.ldb, n0, k_begin, P.N, k_end, P.b_vec, ones_row, tid);
        fa.store(ldsA[0], tid);
        fb.store(ldsB[0], tid);
    }
    __syncthreads();

    for (int kt = 0; kt < nk; ++kt) {
        const int cur = kt & 1;
        if (kt + 1 < nk) {
            const int k0 = k_begin + (kt + 1) * BK;
            fa.load(Ab, P.lda, m0, k0, P.M, k_end, P.a_vec, -1, tid);
            fb.load(Bb, P.ldb, n0, k0, P.N, k_end, P.b_vec, ones_row, tid);
        }
#pragma unroll
        for (int kk = 0; kk < BK / 8; ++kk) {
            float af[FM][4], bf[FN][4];
#pragma unroll
            for (int i = 0; i < FM; ++i) frag_read<BM, BK, LA>(ldsA[cur], wm0 + i * 32 + r, kk, h, af[i]);
#pragma unroll
            for (int j = 0; j < FN; ++j) frag_read<BN, BK, LB>(ldsB[cur], wn0 + j * 32 + r, kk, h, bf[j]);
#pragma unroll
            for (int s = 0; s < 4; ++s)
#pragma unroll
                for (int i = 0; i < FM; ++i)
#pragma unroll
                    for (int j = 0; j < FN; ++j)
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(af[i][s], bf[j][s], acc[i][j], 0, 0, 0);
        }
        if (kt + 1 < nk) {
            fa.store(ldsA[cur ^ 1], tid);
            fb.store(ldsB[cur ^ 1], tid);
        }
        __syncthreads();
    }

    // ---- epilogue: lane holds column n = .. + r and rows 8*(e/4) + 4*h + e%4 of each 32x32 block ----
    float* __restrict__ Cb = P.C + (long long)split * P.split_stride;
#pragma unroll
    for (int j = 0; j < FN; ++j) {
        const int n = n0 + wn0 + j * 32 + r;
        if (n >= P.N) continue;
        float bias = 0.f;
        if (EP == EP_BIAS || EP == EP_BIAS_SIGMOID) bias = P.bias[n];
#pragma unroll
        for (int i = 0; i < FM; ++i) {
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const int m = m0 + wm0 + i * 32 + 8 * (e / 4) + 4 * h + (e % 4);
                if (m >= P.M) continue;
                float x = acc[i][j][e];
                if (EP == EP_BIAS) x += bias;
                if (EP == EP_BIAS_SIGMOID) x = sigmoidf_fast(x + bias);
                if (EP == EP_DSIGMOID) {
                    const float z = P.aux[(long long)(m / P.auxdiv) * P.ldaux + n];
                    x *= z * (1.0f - z);
                }
                Cb[(long long)m * P.ldc + n] = x;
            }
        }
    }
}

}  // namespace dn
