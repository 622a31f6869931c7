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
//
// Pipeline: PF K-tiles are in flight in registers ahead of the tile being multiplied; LDS is
// double-buffered; one barrier per K-tile.  The steady-state loop touches only whole K-tiles and
// has no range checks on k; the ragged last tile goes through a checked loader.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#define DN_MAX_GROUP 8

namespace dn {

typedef float f32x16 __attribute__((ext_vector_type(16)));
// four floats that are only known to be 4-byte aligned
typedef float f32x4u __attribute__((ext_vector_type(4), aligned(4)));

// KC: stored [rows][K], K contiguous.  RC: stored [K][rows], kept row-contiguous in LDS.
// RT: stored [K][rows] like RC, but transposed on the way in: a thread loads four k-consecutive
//     values of one row (each such load is coalesced across the wave, lanes = consecutive rows) and
//     writes them to LDS as one 128-bit store in the KC arrangement, so the MFMA side is identical to KC.
enum OperandLayout { KC = 0, RC = 1, RT = 2 };

// Epilogue of a problem, applied in this order to every output element (m, n):
//   x = alpha * acc;  x += bias[n] (if bias);  x += pre[m * ldpre + n] (if pre);  x = 1/(1+exp(-x)) (if sigmoid);
//   x *= z(1-z) with z = aux[(m / auxdiv) * ldaux + n] (if aux);  x += add[m * ldadd + n] (if add);
//   x += C[m][n] of the same K-slice (if accumulate).

struct GemmProblem {
    const float* A;
    const float* B;
    float* C;
    const float* bias;   // nullable: length N
    const float* aux;    // nullable: activations z whose sigma' = z(1-z) scales the result
    const float* add;    // nullable: matrix added last (may be C itself)
    const float* pre;    // nullable: matrix added before the activation / sigma' scaling (may be C itself)
    long long lda, ldb, ldc, ldaux, ldadd, ldpre;
    float alpha;         // scale of the accumulated product
    int sigmoid;         // 1: logistic function after the bias
    long long split_stride;  // elements between the C outputs of consecutive K-slices
    int M, N, K;
    int auxdiv;          // aux row = output row / auxdiv
    int tiles_m, tiles_n;
    int splits;          // number of K-slices (>= 1)
    int k_per_split;     // multiple of the K tile
    int tile_begin;      // first tile id of this problem within one K-slice of the group
    int b_ones_col;      // 1: column N-1 of op(B) is a virtual column of ones (not read from memory);
                         //    only for a row-contiguous B
    int accumulate;      // 1: the result is added to what C (of the same K-slice) already holds
    int c_rows_padded;   // 1: C has whole tiles of rows (tiles_m * 64), rows past M are padding that may be written
};

struct GemmGroup {
    int nprob;
    int total_tiles;      // tiles_per_split * splits
    int grid;             // work-groups to launch (>= total_tiles)
    int tiles_per_split;  // output tiles of all problems together
    int group_m;          // tile rows per super-row of the tile walk (>= 1)
    int xcd_mode;         // how blockIdx maps to the tile walk, see XcdMode
    GemmProblem p[DN_MAX_GROUP];
};

// The chip has 8 XCDs, each with its own L2; the dispatcher deals work-groups to them round-robin
// (work-group b runs on XCD b % 8; checked on MI355X by reading XCC_ID).  Tiles that share an operand
// panel should therefore not sit at consecutive blockIdx but at blockIdx that are equal modulo 8.
constexpr int kXcds = 8;
// XCD_NONE:    blockIdx is the position in the tile walk.
// XCD_RANGES:  XCD x takes the x-th eighth of the whole walk (launches cut into K-slices: an XCD then
//              reads one slice of the samples, once).
// XCD_PER_PROBLEM: XCD x takes the x-th eighth of every problem's tiles, longest problem first (launches
//              of several problems with different K stay balanced across XCDs).  The grid is padded to
//              8 * (largest per-XCD count); surplus work-groups exit at once.  One K-slice only.
enum XcdMode { XCD_NONE = 0, XCD_RANGES = 1, XCD_PER_PROBLEM = 2 };

__device__ __forceinline__ float sigmoidf_fast(float s) { return 1.0f / (1.0f + __expf(-s)); }

// ---- global -> register tile fetch -------------------------------------------------------
// A tile of an operand is ROWS x BK values.  KC: slot = (row, 4 consecutive k).
// RC: slot = (k, 4 consecutive rows).  Out-of-range elements are zero.  The per-slot address and
// row validity are fixed for the whole K loop and computed once in init().
// Slot modes: 0 nothing to read (zero), 1 four-wide load, 2 element-wise load with row checks,
//             4 four-wide load from a clamped (valid) address; the values land in rows of the tile
//               that lie outside the matrix and never reach memory.
template <int ROWS, int BK, int LAYOUT, int NT>
struct TileFetch {
    static constexpr int SLOTS = ROWS * BK / 4;
    static_assert(SLOTS % NT == 0, "every thread owns whole fetch slots");
    static constexpr int PER_THREAD = SLOTS / NT;
    // LDS strides: KC rows are BK+4 floats apart, RC k-rows are ROWS+8 floats apart.
    static constexpr int LDS_STRIDE = (LAYOUT != RC) ? (BK + 4) : (ROWS + 8);
    static constexpr int LDS_FLOATS = (LAYOUT != RC) ? ROWS * (BK + 4) : BK * (ROWS + 8);

    struct Addr {
        const float* p[PER_THREAD];   // KC: &op[row][4*kq]; RC: &op[0][row]
        int q[PER_THREAD];            // KC: 4*kq (k offset inside the tile); RC: k row inside the tile
        int mode[PER_THREAD];
        int rem[PER_THREAD];          // RC mode 2: valid rows counted from this slot's first row
        int ones_at[PER_THREAD];      // RC mode 2: position (0..3) of the virtual ones row, else -1
        const float* pk[PER_THREAD][4];   // RT: the four k-consecutive elements of the NEXT tile to be loaded
        bool ones[PER_THREAD];        // RT: this slot is the virtual row of ones (its LDS row is written once, by the kernel)
        long long ld;
    };

    // k_first: first k of the first tile that will be loaded (RT keeps running pointers: its loads must be
    // issued tile after tile, in order, which is how the kernel uses them)
    __device__ static __forceinline__ void init(Addr& a, const float* __restrict__ base, long long ld, int row0,
                                                int rows_total, int ones_row, int tid, int k_first) {
        a.ld = ld;
#pragma unroll
        for (int i = 0; i < PER_THREAD; ++i) {
            const int s = tid + i * NT;
            a.mode[i] = 0; a.p[i] = base; a.q[i] = 0; a.rem[i] = 0; a.ones_at[i] = -1; a.ones[i] = false;
#pragma unroll
            for (int e = 0; e < 4; ++e) a.pk[i][e] = base;
            if (LAYOUT == RT) {
                // slot = (row = s % ROWS, four consecutive k starting at 4 * (s / ROWS))
                const int row = row0 + s % ROWS;
                a.q[i] = 4 * (s / ROWS);
                const int real_rows = ones_row >= 0 ? rows_total - 1 : rows_total;  // rows that exist in memory
                // rows past the end, and the virtual row of ones, read the last real row: the former only feed
                // outputs that are never stored, the latter is never stored to LDS (see store_one())
                const int rr = row < real_rows ? row : real_rows - 1;
                a.ones[i] = row == ones_row;
                a.mode[i] = row < real_rows ? 1 : 4;
#pragma unroll
                for (int e = 0; e < 4; ++e) a.pk[i][e] = base + (long long)(k_first + a.q[i] + e) * ld + rr;
            } else if (LAYOUT == KC) {
                const int row = row0 + s / (BK / 4);
                a.q[i] = 4 * (s % (BK / 4));
                // rows past the end read the last valid row
                const int rr = row < rows_total ? row : rows_total - 1;
                a.p[i] = base + (long long)rr * ld + a.q[i];
                a.mode[i] = row < rows_total ? 1 : 4;
            } else {
                const int row = row0 + 4 * (s % (ROWS / 4));
                a.q[i] = s / (ROWS / 4);
                const int real_rows = ones_row >= 0 ? rows_total - 1 : rows_total;  // rows that exist in memory
                if (row + 3 < real_rows) {
                    a.p[i] = base + row;
                    a.mode[i] = 1;
                } else if (row < rows_total) {
                    a.p[i] = base + row;
                    a.rem[i] = rows_total - row;
                    if (ones_row >= row && ones_row <= row + 3) a.ones_at[i] = ones_row - row;
                    a.mode[i] = 2;
                } else if (real_rows >= 4) {
                    a.p[i] = base;          // any valid address; result discarded
                    a.mode[i] = 4;
                }
            }
        }
    }

    float4 v[PER_THREAD];

    __device__ __forceinline__ void rc_elements(const Addr& a, int i, const float* p, float4& x) const {
        if (a.rem[i] > 0) x.x = (a.ones_at[i] == 0) ? 1.f : p[0];
        if (a.rem[i] > 1) x.y = (a.ones_at[i] == 1) ? 1.f : p[1];
        if (a.rem[i] > 2) x.z = (a.ones_at[i] == 2) ? 1.f : p[2];
        if (a.rem[i] > 3) x.w = (a.ones_at[i] == 3) ? 1.f : p[3];
    }

    // RT: the slot's four values of the next tile; the pointers move on by one tile (one 64-bit add each,
    // instead of a 64-bit multiply-add and three adds from scratch per slot and tile)
    __device__ static __forceinline__ float4 rt_next(Addr& a, int i) {
        const float4 x = make_float4(*a.pk[i][0], *a.pk[i][1], *a.pk[i][2], *a.pk[i][3]);
#pragma unroll
        for (int e = 0; e < 4; ++e) a.pk[i][e] += (long long)BK * a.ld;
        return x;
    }

    // Tile lies entirely below k_end: no k checks.  Vector loads only assume 4-byte alignment
    // (f32x4u); the compiler picks the widest access the target allows for that.
    __device__ __forceinline__ void load_full(Addr& a, int k0) {
#pragma unroll
        for (int i = 0; i < PER_THREAD; ++i) {
            float4 x = make_float4(0.f, 0.f, 0.f, 0.f);
            if (LAYOUT == RT) {
                x = rt_next(a, i);
            } else if (LAYOUT == KC) {
                const f32x4u t = *reinterpret_cast<const f32x4u*>(a.p[i] + k0);
                x = make_float4(t[0], t[1], t[2], t[3]);
            } else {
                const float* p = a.p[i] + (long long)(k0 + a.q[i]) * a.ld;
                if (a.mode[i] == 1 || a.mode[i] == 4) {
                    const f32x4u t = *reinterpret_cast<const f32x4u*>(p);
                    x = make_float4(t[0], t[1], t[2], t[3]);
                } else if (a.mode[i] == 2) {
                    rc_elements(a, i, p, x);
                }
            }
            v[i] = x;
        }
    }

    // One slot of a whole tile whose slots are all of mode 1 or 4 (checked once per work-group).
    __device__ __forceinline__ void load_clean_one(Addr& a, int k0, int i) {
        if (LAYOUT == RT) {
            v[i] = rt_next(a, i);
        } else {
            const float* p = (LAYOUT == KC) ? a.p[i] + k0 : a.p[i] + (long long)(k0 + a.q[i]) * a.ld;
            const f32x4u t = *reinterpret_cast<const f32x4u*>(p);
            v[i] = make_float4(t[0], t[1], t[2], t[3]);
        }
    }

    __device__ __forceinline__ void store_one(const Addr& a, float* lds, int tid, int i) const {
        if (LAYOUT == RT && a.ones[i]) return;      // that LDS row holds ones for good
        *reinterpret_cast<float4*>(lds + lds_offset(tid + i * NT)) = v[i];
    }

    __device__ static __forceinline__ int lds_offset(int s) {
        if (LAYOUT == KC) return (s / (BK / 4)) * LDS_STRIDE + 4 * (s % (BK / 4));
        if (LAYOUT == RT) return (s % ROWS) * LDS_STRIDE + 4 * (s / ROWS);
        return (s / (ROWS / 4)) * LDS_STRIDE + 4 * (s % (ROWS / 4));
    }

    __device__ static __forceinline__ bool all_clean(const Addr& a) {
        bool ok = true;
#pragma unroll
        for (int i = 0; i < PER_THREAD; ++i) ok = ok && (a.mode[i] == 1 || a.mode[i] == 4);
        return ok;
    }

    // Last, partial K tile: every element is checked against k_end.
    __device__ __forceinline__ void load_tail(Addr& a, int k0, int k_end) {
#pragma unroll
        for (int i = 0; i < PER_THREAD; ++i) {
            float4 x = make_float4(0.f, 0.f, 0.f, 0.f);
            if (LAYOUT == RT) {
                const int k = k0 + a.q[i];
                if (k + 0 < k_end) x.x = *a.pk[i][0];
                if (k + 1 < k_end) x.y = *a.pk[i][1];
                if (k + 2 < k_end) x.z = *a.pk[i][2];
                if (k + 3 < k_end) x.w = *a.pk[i][3];
#pragma unroll
                for (int e = 0; e < 4; ++e) a.pk[i][e] += (long long)BK * a.ld;
            } else if (LAYOUT == KC) {
                const int k = k0 + a.q[i];
                const float* p = a.p[i] + k0;
                if (a.mode[i] == 1) {
                    if (k + 0 < k_end) x.x = p[0];
                    if (k + 1 < k_end) x.y = p[1];
                    if (k + 2 < k_end) x.z = p[2];
                    if (k + 3 < k_end) x.w = p[3];
                }
            } else {
                const int k = k0 + a.q[i];
                if (k < k_end) {
                    const float* p = a.p[i] + (long long)k * a.ld;
                    if (a.mode[i] == 1) {
                        const f32x4u t = *reinterpret_cast<const f32x4u*>(p);
                        x = make_float4(t[0], t[1], t[2], t[3]);
                    } else if (a.mode[i] == 2) {
                        rc_elements(a, i, p, x);
                    }
                }
            }
            v[i] = x;
        }
    }

    // Slots of mode 4 carry the values of some other, valid row.  They only ever feed output rows
    // (or columns) beyond M (or N), which the epilogue never writes, so they need no zeroing.
    __device__ __forceinline__ void store(const Addr& a, float* lds, int tid) const {
#pragma unroll
        for (int i = 0; i < PER_THREAD; ++i) store_one(a, lds, tid, i);
    }

    // RT with a virtual row of ones inside this tile: fill that row of an LDS buffer (all threads call this
    // once per buffer, before the first barrier; the row is never stored to afterwards)
    __device__ static __forceinline__ void fill_ones_row(float* lds, int local_row, int tid) {
        if (LAYOUT == RT && local_row >= 0 && local_row < ROWS)
            for (int k = tid; k < BK; k += NT) lds[local_row * LDS_STRIDE + k] = 1.0f;
    }
};

// Fetch the four k-step values of one 32-row MFMA operand block for k-group kk (8 k values).
template <int ROWS, int BK, int LAYOUT>
__device__ __forceinline__ void frag_read(const float* lds, int row, int kk, int h, float (&f)[4]) {
    if (LAYOUT != RC) {
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
// PF = number of K tiles kept in flight in registers ahead of the one being multiplied.
// PIN = use the hand-interleaved steady-state loop.
// CLS = caller's kernel-class number; it changes no code, only the symbol, so that a profiler's
//       per-kernel statistics separate the call sites (forward, back-propagation, sweeps, products...).
// Tiles of 128 x 128 are compiled for two work-groups per CU (at most 256 registers): alone on a CU a work-group's
// epilogue (sigmoid, or the sigma' scaling with its extra loads) leaves the matrix pipes idle, which costs up to 9 % of
// the launch (2000000 x 4096 x 4096 with the sigma' scaling: 518 ms with one work-group per CU, 476 ms with two).
template <int BM, int BN, int BK, int WGM, int WGN, int LA, int LB, int PF, bool PIN, int CLS>
__global__ __launch_bounds__(256, (BM * BN >= 128 * 128 ? 2 : 1)) void gemm_kernel(const GemmGroup g) {
    constexpr int NT = 256;
    static_assert(WGM * WGN == 4, "four waves per work-group");
    constexpr int WM = BM / WGM, WN = BN / WGN;
    constexpr int FM = WM / 32, FN = WN / 32;
    static_assert(WM % 32 == 0 && WN % 32 == 0 && BK % 8 == 0, "tile shape");
    static_assert(PF % 2 == 0 && PF >= 2 && PF <= 8, "prefetch depth must be even so LDS buffer parity is static");
    using FetchA = TileFetch<BM, BK, LA, NT>;
    using FetchB = TileFetch<BN, BK, LB, NT>;

    __shared__ __attribute__((aligned(16))) float ldsA[2][FetchA::LDS_FLOATS];
    __shared__ __attribute__((aligned(16))) float ldsB[2][FetchB::LDS_FLOATS];

    // ---- which problem / tile / K-slice ----
    // Tile walk (logical ids): K-slice outermost, then problem, then super-rows of group_m tile rows,
    // inside a super-row down the rows first.  A contiguous stretch of the walk is a compact patch of
    // the output (its tiles share A and B panels) inside one K-slice (its tiles read the same rows of
    // both operands of a sum over samples).  XCD x takes the x-th eighth of the walk, so that sharing
    // happens inside one L2.
    int lid = blockIdx.x;
    int split = 0, t = 0, pi = 0;
    if (g.xcd_mode == XCD_PER_PROBLEM) {
        const int x = lid % kXcds;
        int kx = lid / kXcds;
        pi = -1;
#pragma unroll
        for (int i = 0; i < DN_MAX_GROUP; ++i) {
            if (i < g.nprob && pi < 0) {
                const int tiles = g.p[i].tiles_m * g.p[i].tiles_n;
                const int per = tiles / kXcds, rem = tiles % kXcds;
                const int mine = per + (x < rem ? 1 : 0);
                if (kx < mine) { pi = i; t = x * per + min(x, rem) + kx; }
                else kx -= mine;
            }
        }
        if (pi < 0) return;      // padding work-group
    } else {
        if (g.xcd_mode == XCD_RANGES) {
            const int x = lid % kXcds, kx = lid / kXcds;
            const int per = g.total_tiles / kXcds, rem = g.total_tiles % kXcds;
            lid = x * per + min(x, rem) + kx;
        }
        split = lid / g.tiles_per_split;
        t = lid - split * g.tiles_per_split;
#pragma unroll
        for (int i = 1; i < DN_MAX_GROUP; ++i)
            if (i < g.nprob && t >= g.p[i].tile_begin) pi = i;
        t -= g.p[pi].tile_begin;
    }
    const GemmProblem& P = g.p[pi];
    const int per_group = g.group_m * P.tiles_n;
    const int grp = t / per_group;
    const int first_tm = grp * g.group_m;
    const int gsz = min(P.tiles_m - first_tm, g.group_m);
    const int tg = t - grp * per_group;
    const int tm = first_tm + tg % gsz;
    const int tn = tg / gsz;
    const int m0 = tm * BM, n0 = tn * BN;
    const int k_begin = split * P.k_per_split;
    const int k_end = min(P.K, k_begin + P.k_per_split);

    const int tid = threadIdx.x;
    const int wave = tid >> 6, lane = tid & 63;
    const int r = lane & 31, h = lane >> 5;
    const int wm0 = (wave / WGN) * WM, wn0 = (wave % WGN) * WN;

    const int ones_row = P.b_ones_col ? (P.N - 1) : -1;

    f32x16 acc[FM][FN];
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

    typename FetchA::Addr aa;
    typename FetchB::Addr ab;
    FetchA::init(aa, P.A, P.lda, m0, P.M, -1, tid, k_begin);
    FetchB::init(ab, P.B, P.ldb, n0, P.N, ones_row, tid, k_begin);
    FetchA fa[PF];
    FetchB fb[PF];
    if (LB == RT && ones_row >= 0) {
        FetchB::fill_ones_row(ldsB[0], ones_row - n0, tid);
        FetchB::fill_ones_row(ldsB[1], ones_row - n0, tid);
    }

    const int klen = max(k_end - k_begin, 0);
    const int nfull = klen / BK;                    // whole K tiles
    const int nk = nfull + ((klen - nfull * BK) > 0 ? 1 : 0);

    auto fetch = [&](int slot, int kt) {
        // kt < nk is guaranteed by the callers
        const int k0 = k_begin + kt * BK;
        if (kt < nfull) { fa[slot].load_full(aa, k0); fb[slot].load_full(ab, k0); }
        else            { fa[slot].load_tail(aa, k0, k_end); fb[slot].load_tail(ab, k0, k_end); }
    };
    // Fragment reads run one k-group ahead of the MFMAs that use them, so the LDS latency of group
    // kk+1 is covered by the MFMAs of group kk.
    auto multiply = [&](int cur) {
        constexpr int KG = BK / 8;
        float af[2][FM][4], bf[2][FN][4];
#pragma unroll
        for (int i = 0; i < FM; ++i) frag_read<BM, BK, LA>(ldsA[cur], wm0 + i * 32 + r, 0, h, af[0][i]);
#pragma unroll
        for (int j = 0; j < FN; ++j) frag_read<BN, BK, LB>(ldsB[cur], wn0 + j * 32 + r, 0, h, bf[0][j]);
#pragma unroll
        for (int kk = 0; kk < KG; ++kk) {
            const int cb = kk & 1;
            if (kk + 1 < KG) {
#pragma unroll
                for (int i = 0; i < FM; ++i)
                    frag_read<BM, BK, LA>(ldsA[cur], wm0 + i * 32 + r, kk + 1, h, af[cb ^ 1][i]);
#pragma unroll
                for (int j = 0; j < FN; ++j)
                    frag_read<BN, BK, LB>(ldsB[cur], wn0 + j * 32 + r, kk + 1, h, bf[cb ^ 1][j]);
            }
#pragma unroll
            for (int s4 = 0; s4 < 4; ++s4)
#pragma unroll
                for (int i = 0; i < FM; ++i)
#pragma unroll
                    for (int j = 0; j < FN; ++j)
                        acc[i][j] =
                            __builtin_amdgcn_mfma_f32_32x32x2f32(af[cb][i][s4], bf[cb][j][s4], acc[i][j], 0, 0, 0);
        }
    };

    // prologue: tiles 0..PF-1 into registers, tile 0 into LDS
    if (nfull >= PF) {
        // common case, kept free of the checked loader so the PF tiles are issued back to back
#pragma unroll
        for (int u = 0; u < PF; ++u) {
            fa[u].load_full(aa, k_begin + u * BK);
            fb[u].load_full(ab, k_begin + u * BK);
        }
    } else {
#pragma unroll
        for (int u = 0; u < PF; ++u)
            if (u < nk) fetch(u, u);
    }
    if (nk > 0) {
        fa[0].store(aa, ldsA[0], tid);
        fb[0].store(ab, ldsB[0], tid);
    }
    __syncthreads();

    // Long contractions are summed in segments of kFlushTiles K-tiles: the MFMA accumulator is folded
    // into a second fp32 accumulator and cleared, which shortens the chains of dependent fp32 roundings
    // (error grows with the square root of the chain length).
    f32x16 acc2[FM][FN];
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc2[i][j][e] = 0.f;
    constexpr int kFlushTiles = 512 / BK;
    int since_flush = 0;

    int kt0 = 0;
    // ---- steady state -------------------------------------------------------------------------
    // Entered only by work-groups whose fetch slots are all plain four-wide loads (no ragged rows, no
    // virtual column in this tile); the others do all their tiles in the checked loop below.
    // A wave issues in order, so a memory instruction only overlaps the matrix pipe if it sits
    // between two MFMAs.  Each K-tile is therefore laid out by hand as
    //     [LDS reads of k-group 0]
    //     {MFMA of the previous tile's last k-group} x {LDS writes of tile kt+1, global loads of tile kt+PF}
    //     {MFMA of k-group g} x {LDS reads of k-group g+1, remaining writes/loads}     g = 0..KG-2
    //     [barrier]
    // with one memory instruction after each MFMA and scheduling fences that keep the compiler from
    // regrouping them.  The last k-group of a tile is multiplied after the barrier, which covers the
    // LDS latency of the next tile's first reads.
    // Measured: the hand-placed order (PIN) wins when a launch has few work-groups per CU, so that a wave
    // has little company on its SIMD, and both operands are K-contiguous (few, wide LDS reads); with many
    // resident waves, or with row-contiguous operands (four narrow LDS reads per fragment), the compiler's
    // own schedule of the plain loop below is as good or better.  The host picks per launch.
    constexpr bool kPinned = PIN;
    const bool clean = __syncthreads_and((FetchA::all_clean(aa) && FetchB::all_clean(ab)) ? 1 : 0) != 0;
    if (!kPinned) {
        // plain steady state: whole tiles only, no k checks, compiler-scheduled
        for (; kt0 + 2 * PF <= nfull; kt0 += PF) {
            if (since_flush >= kFlushTiles) {
                since_flush = 0;
#pragma unroll
                for (int i = 0; i < FM; ++i)
#pragma unroll
                    for (int j = 0; j < FN; ++j)
#pragma unroll
                        for (int e = 0; e < 16; ++e) {
                            acc2[i][j][e] += acc[i][j][e];
                            acc[i][j][e] = 0.f;
                        }
            }
            since_flush += PF;
#pragma unroll
            for (int u = 0; u < PF; ++u) {
                // register slot u held tile kt0+u, which already sits in LDS: refill it with tile kt0+u+PF
                const int k0 = k_begin + (kt0 + u + PF) * BK;
                fa[u].load_full(aa, k0);
                fb[u].load_full(ab, k0);
                multiply(u & 1);                 // u & 1 == kt & 1 because PF is even
                fa[(u + 1) % PF].store(aa, ldsA[(u & 1) ^ 1], tid);
                fb[(u + 1) % PF].store(ab, ldsB[(u & 1) ^ 1], tid);
                __syncthreads();
            }
        }
    } else if (clean && 2 * PF <= nfull) {
        constexpr int KG = BK / 8;
        constexpr int NA = FetchA::PER_THREAD, NB = FetchB::PER_THREAD;
        constexpr int NOPS = 2 * (NA + NB);
        float daf[FM][4], dbf[FN][4];          // fragments of the deferred k-group
#pragma unroll
        for (int i = 0; i < FM; ++i)
#pragma unroll
            for (int c = 0; c < 4; ++c) daf[i][c] = 0.f;
#pragma unroll
        for (int j = 0; j < FN; ++j)
#pragma unroll
            for (int c = 0; c < 4; ++c) dbf[j][c] = 0.f;

        for (; kt0 + 2 * PF <= nfull; kt0 += PF) {
            if (since_flush >= kFlushTiles) {
                since_flush = 0;
#pragma unroll
                for (int i = 0; i < FM; ++i)
#pragma unroll
                    for (int j = 0; j < FN; ++j)
#pragma unroll
                        for (int e = 0; e < 16; ++e) {
                            acc2[i][j][e] += acc[i][j][e];
                            acc[i][j][e] = 0.f;
                        }
            }
            since_flush += PF;
#pragma unroll
            for (int u = 0; u < PF; ++u) {
                const int cur = u & 1;                      // == kt & 1 because PF is even
                const int k0 = k_begin + (kt0 + u + PF) * BK;
                const float* la = ldsA[cur];
                const float* lb = ldsB[cur];
                // memory instruction number `op` of this tile: stores of slot u+1 first, then refills of slot u
                auto mem_op = [&](int op) {
                    if (op < NA)               fa[(u + 1) % PF].store_one(aa, ldsA[cur ^ 1], tid, op);
                    else if (op < NA + NB)     fb[(u + 1) % PF].store_one(ab, ldsB[cur ^ 1], tid, op - NA);
                    else if (op < 2 * NA + NB) fa[u].load_clean_one(aa, k0, op - NA - NB);
                    else if (op < NOPS)        fb[u].load_clean_one(ab, k0, op - 2 * NA - NB);
                };
                float af[2][FM][4], bf[2][FN][4];
#pragma unroll
                for (int i = 0; i < FM; ++i) frag_read<BM, BK, LA>(la, wm0 + i * 32 + r, 0, h, af[0][i]);
#pragma unroll
                for (int j = 0; j < FN; ++j) frag_read<BN, BK, LB>(lb, wn0 + j * 32 + r, 0, h, bf[0][j]);
                __builtin_amdgcn_sched_barrier(0);
                int op = 0;
                // deferred k-group of the previous tile
#pragma unroll
                for (int s4 = 0; s4 < 4; ++s4)
#pragma unroll
                    for (int i = 0; i < FM; ++i)
#pragma unroll
                        for (int j = 0; j < FN; ++j) {
                            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(daf[i][s4], dbf[j][s4], acc[i][j], 0, 0, 0);
                            mem_op(op++);
                            __builtin_amdgcn_sched_barrier(0);
                        }
                // k-groups 0 .. KG-2 of this tile, reading the next group's fragments on the way
#pragma unroll
                for (int kk = 0; kk + 1 < KG; ++kk) {
                    const int cb = kk & 1;
                    int rd = 0;
#pragma unroll
                    for (int s4 = 0; s4 < 4; ++s4)
#pragma unroll
                        for (int i = 0; i < FM; ++i)
#pragma unroll
                            for (int j = 0; j < FN; ++j) {
                                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(af[cb][i][s4], bf[cb][j][s4],
                                                                                 acc[i][j], 0, 0, 0);
                                if (rd < FM)
                                    frag_read<BM, BK, LA>(la, wm0 + rd * 32 + r, kk + 1, h, af[cb ^ 1][rd]);
                                else if (rd < FM + FN)
                                    frag_read<BN, BK, LB>(lb, wn0 + (rd - FM) * 32 + r, kk + 1, h, bf[cb ^ 1][rd - FM]);
                                else
                                    mem_op(op++);
                                ++rd;
                                __builtin_amdgcn_sched_barrier(0);
                            }
                }
                // whatever did not fit between MFMAs
#pragma unroll
                for (int rest = 0; rest < NOPS; ++rest)
                    if (rest >= op) mem_op(rest);
                // the last k-group waits until after the barrier
#pragma unroll
                for (int i = 0; i < FM; ++i)
#pragma unroll
                    for (int c = 0; c < 4; ++c) daf[i][c] = af[(KG - 1) & 1][i][c];
#pragma unroll
                for (int j = 0; j < FN; ++j)
#pragma unroll
                    for (int c = 0; c < 4; ++c) dbf[j][c] = bf[(KG - 1) & 1][j][c];
                __syncthreads();
            }
        }
        // the deferred k-group of the last steady-state tile
#pragma unroll
        for (int s4 = 0; s4 < 4; ++s4)
#pragma unroll
            for (int i = 0; i < FM; ++i)
#pragma unroll
                for (int j = 0; j < FN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(daf[i][s4], dbf[j][s4], acc[i][j], 0, 0, 0);
    }
    // checked loop: the tiles the steady state did not take; refills stop at nk, the last tile may be
    // ragged, slots may need element-wise loads
    for (; kt0 < nk; kt0 += PF) {
        if (since_flush >= kFlushTiles) {
            since_flush = 0;
#pragma unroll
            for (int i = 0; i < FM; ++i)
#pragma unroll
                for (int j = 0; j < FN; ++j)
#pragma unroll
                    for (int e = 0; e < 16; ++e) {
                        acc2[i][j][e] += acc[i][j][e];
                        acc[i][j][e] = 0.f;
                    }
        }
        since_flush += PF;
#pragma unroll
        for (int u = 0; u < PF; ++u) {
            const int kt = kt0 + u;
            if (kt < nk) {
                if (kt + PF < nk) fetch(u, kt + PF);
                multiply(u & 1);
                if (kt + 1 < nk) {
                    fa[(u + 1) % PF].store(aa, ldsA[(u & 1) ^ 1], tid);
                    fb[(u + 1) % PF].store(ab, ldsB[(u & 1) ^ 1], tid);
                }
                __syncthreads();
            }
        }
    }

    // ---- epilogue: lane holds column n = .. + r and rows 8*(e/4) + 4*h + e%4 of each 32x32 block ----
    // Tiles of 20-50 K-steps spend a tenth of their time here, so the common cases are kept lean: one 64-bit
    // pointer per operand and block (row offsets are multiples of the leading dimension, uniform), no row checks
    // when the whole tile lies inside the matrix (uniform test), and a branch-free body when nothing but alpha
    // and the bias apply.
    float* __restrict__ Cb = P.C + (long long)split * P.split_stride;
    const bool plain = !P.sigmoid && !P.aux && !P.add && !P.accumulate && !P.pre;   // uniform
    const bool full_rows = m0 + BM <= P.M || P.c_rows_padded;                          // uniform
    const float alpha = P.alpha;
#pragma unroll
    for (int j = 0; j < FN; ++j) {
        const int n = n0 + wn0 + j * 32 + r;
        if (n >= P.N) continue;
        const float bias = P.bias ? P.bias[n] : 0.f;
#pragma unroll
        for (int i = 0; i < FM; ++i) {
            const int mb = m0 + wm0 + i * 32 + 4 * h;            // row of element e = 0
            const int mleft = P.M - mb;                          // rows from mb on that exist
            float* __restrict__ cp = Cb + (long long)mb * P.ldc + n;
            if (plain) {
                if (full_rows) {
#pragma unroll
                    for (int e = 0; e < 16; ++e)
                        cp[(long long)(8 * (e / 4) + (e % 4)) * P.ldc] = alpha * (acc[i][j][e] + acc2[i][j][e]) + bias;
                } else {
#pragma unroll
                    for (int e = 0; e < 16; ++e)
                        if (8 * (e / 4) + (e % 4) < mleft)
                            cp[(long long)(8 * (e / 4) + (e % 4)) * P.ldc] = alpha * (acc[i][j][e] + acc2[i][j][e]) + bias;
                }
            } else {
                const float* __restrict__ prep = P.pre ? P.pre + (long long)mb * P.ldpre + n : nullptr;
                const float* __restrict__ addp = P.add ? P.add + (long long)mb * P.ldadd + n : nullptr;
                // activation row of output row mb + dm: one division per block of 32 rows instead of one per element
                // (the 28 rows a lane holds cross a multiple of auxdiv at most once when auxdiv >= 28)
                const int aux_q = P.aux ? mb / P.auxdiv : 0;
                const int aux_r = P.aux ? mb - aux_q * P.auxdiv : 0;
                const bool aux_fast = P.auxdiv >= 28;                                          // uniform
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    const int dm = 8 * (e / 4) + (e % 4);
                    if (!full_rows && dm >= mleft) continue;
                    float x = alpha * (acc[i][j][e] + acc2[i][j][e]) + bias;
                    if (prep) x += prep[(long long)dm * P.ldpre];
                    if (P.sigmoid) x = sigmoidf_fast(x);
                    if (P.aux) {
                        const int arow = P.auxdiv == 1 ? mb + dm
                                         : aux_fast    ? aux_q + (aux_r + dm >= P.auxdiv ? 1 : 0)
                                                       : (mb + dm) / P.auxdiv;
                        const float z = P.aux[(long long)arow * P.ldaux + n];
                        x *= z * (1.0f - z);
                    }
                    if (addp) x += addp[(long long)dm * P.ldadd];
                    if (P.accumulate) x += cp[(long long)dm * P.ldc];
                    cp[(long long)dm * P.ldc] = x;
                }
            }
        }
    }
}

}  // namespace dn
