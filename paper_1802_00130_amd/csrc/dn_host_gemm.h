// Launch plumbing of the GEMM engine: problem descriptors, tile walk, tile and K-slice choices.
// Part of the one translation unit dn_lib.hip (helpers live in its unnamed namespace).
#pragma once
#include "dn_host_ctx.h"

namespace {

// ---- GEMM plumbing -----------------------------------------------------------------------

GemmProblem mk_problem(const float* A, long long lda, const float* B, long long ldb, float* Cc, long long ldc, int M,
                       int N, int K) {
    GemmProblem p;
    std::memset(&p, 0, sizeof(p));
    p.A = A; p.B = B; p.C = Cc;
    p.lda = lda; p.ldb = ldb; p.ldc = ldc;
    p.M = M; p.N = N; p.K = K;
    p.auxdiv = 1;
    p.alpha = 1.0f;
    p.splits = 1;
    p.k_per_split = K;
    return p;
}

// Floats of one K-slice of layer m's partial sums over samples: rows padded to whole 64-row tiles, so that the
// products that write them need no row checks (the fold reads the first n_m rows only).
long long tn_slice_floats(const dn_ctx* c, int m) { return round_up(c->dims[m], 64) * c->ldw[m]; }

// Fill tile counts and the tile walk.  splits applies to every problem of the group.
void finalize_group(GemmGroup& g, int BM, int BN, int BK, int splits) {
    int begin = 0;
    for (int i = 0; i < g.nprob; ++i) {
        GemmProblem& p = g.p[i];
        p.tiles_m = cdiv(p.M, BM);
        p.tiles_n = cdiv(p.N, BN);
        p.splits = splits;
        p.k_per_split = (int)round_up(cdiv(p.K, splits), BK);
        p.tile_begin = begin;
        begin += p.tiles_m * p.tiles_n;
    }
    g.tiles_per_split = begin;
    g.total_tiles = begin * splits;
    g.group_m = kGroupM;
    g.grid = g.total_tiles;
    if (splits > 1 || g.nprob == 1) {
        g.xcd_mode = XCD_RANGES;
    } else {
        g.xcd_mode = XCD_PER_PROBLEM;
        int most = 0;
        for (int x = 0; x < kXcds; ++x) {
            int mine = 0;
            for (int i = 0; i < g.nprob; ++i) {
                const int tiles = g.p[i].tiles_m * g.p[i].tiles_n;
                mine += tiles / kXcds + (x < tiles % kXcds ? 1 : 0);
            }
            most = std::max(most, mine);
        }
        g.grid = kXcds * most;
    }
}

int group_tiles(const GemmGroup& g, int BM, int BN) {
    int t = 0;
    for (int i = 0; i < g.nprob; ++i) t += cdiv(g.p[i].M, BM) * cdiv(g.p[i].N, BN);
    return t;
}

template <int BM, int BN, int BK, int PF, int LA, int LB, int CLS, bool PIN = false>
hipError_t launch_gemm_t(const GemmGroup& g, hipStream_t st) {
    if (g.total_tiles <= 0) return hipSuccess;
    hipLaunchKernelGGL((gemm_kernel<BM, BN, BK, 2, 2, LA, LB, PF, PIN, CLS>), dim3(g.grid), dim3(256), 0, st, g);
    return hipGetLastError();
}

// 64x64 tiles, K-tile 16, 4 K-tiles in flight (2 for short sums and for sums over samples).  The hand-placed
// schedule is used for launches of at most 4 work-groups per CU and, at every size, when both operands go through
// the transposing loads (sums over samples); elsewhere the compiler's schedule of the plain loop is as good.
// 128x128 tiles (64x64 per wave: half the LDS and L2 traffic per flop; two work-groups per CU, hand-placed schedule)
// pay when the launch fills whole rounds of work-groups and loses little to padding: measured stand-alone against
// the 64x64 tiles with K-tiles of 32, 200000 x 4096 x 4096 132 -> 142 TFLOP/s (130 -> 141 with the sigma' scaling),
// 100000 x 2000 x 2000 with bias and sigmoid 119 -> 133, 2000 x 4096 x 4096 (512 tiles) 126 -> 137, but 5000 x 2000 x 2048
// (640 tiles: two and a half rounds of 256) 124 -> 110.  In the step (4096 x 5 - 1000): forward 219 -> 204 ms, gradient
// 627 -> 600 ms, Jacobian sweeps 1548 -> 1437 ms; 2048-2000-2000-2000-100: 21.1 -> 19.1, 63.9 -> 56.6, 73.5 -> 63.3 ms.
// `only`: bit i set = problem i takes part (all by default).
bool prefer_128(const GemmGroup& g, unsigned only = ~0u) {
    double steps128 = 0.0, steps64 = 0.0;      // in K-tile steps of a 64x64 tile
    long long t128 = 0;
    for (int i = 0; i < g.nprob; ++i) {
        if (!((only >> i) & 1u)) continue;
        const GemmProblem& p = g.p[i];
        const long long a = (long long)cdiv(p.M, 128) * cdiv(p.N, 128), b = (long long)cdiv(p.M, 64) * cdiv(p.N, 64);
        t128 += a;
        steps128 += 4.0 * (double)a * cdiv(p.K, 16);
        steps64 += (double)b * cdiv(p.K, 16);
    }
    if (t128 < 2 * 256) return false;
    const double rounds = (double)cdiv(t128, 256);
    const double fill = (double)t128 / (256.0 * rounds);
    return steps128 / (fill * 1.08) < 0.97 * steps64;
}

// Which problems of a group go through the large tiles: all of them if the whole group passes the test above;
// else the problems with at least a round of large tiles each, if they pass it among themselves (the rest then
// gets a launch of small tiles of its own: the inner sums of 4096 x 5 - 1000 over 2000 samples are four layers of 512
// large tiles, exactly four rounds, and a fifth of 128, which as small tiles costs 0.15 ms instead of a fifth round:
// 2.43 -> 2.32 ms); else none.
unsigned pick_128(const GemmGroup& g) {
    const unsigned all = g.nprob >= 32 ? ~0u : ((1u << g.nprob) - 1u);
    if (prefer_128(g, all)) return all;
    unsigned big = 0;
    for (int i = 0; i < g.nprob; ++i)
        if ((long long)cdiv(g.p[i].M, 128) * cdiv(g.p[i].N, 128) >= 256) big |= 1u << i;
    if (big != 0 && big != all && prefer_128(g, big)) return big;
    return 0;
}

template <int LA, int LB, int CLS>
hipError_t launch_gemm(GemmGroup& g, int splits, hipStream_t st) {
    // sums over samples (both operands through the transposing loads): two K-tiles in flight (measured 4-6 % faster
    // than four at every shape: 300 x 785 x 3000 in 8 slices 30.0 -> 28.2 us, 1024 x 1024 x 60000 1157 -> 1097 us)
    if (LA == RT || LB == RT) finalize_group(g, 64, 64, 16, splits);
    if (LA == RT && LB == RT) return launch_gemm_t<64, 64, 16, 2, LA, LB, CLS, true>(g, st);
    // sums over samples whose right operand was transposed beforehand (the products): the same schedule; one operand
    // through the transposing loads leaves room for a fourth work-group per CU and is 3-9 % faster at every shape
    // (4096 x 4097 x 2000: 595 -> 565 us, 1000 x 3073 x 2500: 187 -> 171 us, 300 x 785 x 3000 in 8 slices 26.7 -> 25.6 us)
    if (LA == RT && LB == KC) return launch_gemm_t<64, 64, 16, 2, LA, LB, CLS, true>(g, st);
    if (LA == KC && LB == KC && splits == 1) {
        const unsigned large = pick_128(g);
        if (large != 0) {
            GemmGroup a, b;
            a.nprob = b.nprob = 0;
            for (int i = 0; i < g.nprob; ++i) {
                if ((large >> i) & 1u) a.p[a.nprob++] = g.p[i];
                else                   b.p[b.nprob++] = g.p[i];
            }
            finalize_group(a, 128, 128, 16, splits);
            const hipError_t e = launch_gemm_t<128, 128, 16, 2, LA, LB, CLS, true>(a, st);
            if (e != hipSuccess || b.nprob == 0) return e;
            g = b;      // the rest: small tiles, chosen below
        }
    }
    finalize_group(g, 64, 64, 16, splits);
    if (g.total_tiles <= 4 * 256) return launch_gemm_t<64, 64, 16, 4, LA, LB, CLS, true>(g, st);
    // short sums (K <= 1024): two K-tiles in flight are enough, and the smaller register footprint lets a fifth
    // work-group onto each CU (60000 x 300 x 300: 119 -> 113 us)
    int kmax = 0;
    for (int i = 0; i < g.nprob; ++i) kmax = std::max(kmax, g.p[i].K);
    if (kmax <= 1024) return launch_gemm_t<64, 64, 16, 2, LA, LB, CLS>(g, st);
    // long sums over K-contiguous operands: K-tiles of 32, two in flight (half the barriers per flop;
    // 50000 x 1000 x 3072: 121 -> 127 TFLOP/s, 60000 x 4096 x 4096: 125 -> 132, 120000 x 2000 x 2000: 120 -> 122;
    // no gain at K = 1000 and a loss below that, and a large loss with the transposing loads)
    if (LA == KC && LB == KC && splits == 1) {
        long long heaviest = -1;
        int k_heavy = 0;
        for (int i = 0; i < g.nprob; ++i) {
            const long long w = (long long)g.p[i].tiles_m * g.p[i].tiles_n * g.p[i].K;
            if (w > heaviest) { heaviest = w; k_heavy = g.p[i].K; }
        }
        if (k_heavy >= 2000) {
            finalize_group(g, 64, 64, 32, splits);
            return launch_gemm_t<64, 64, 32, 2, LA, LB, CLS>(g, st);
        }
    }
    return launch_gemm_t<64, 64, 16, 4, LA, LB, CLS>(g, st);
}

// K-slices of a sum over samples (64x64 tiles, both operands through the transposing loads), at least 256
// samples per slice.  That kernel keeps 3 work-groups on a CU, 768 on the chip; work-groups beyond a multiple
// of 768 run a further round on nearly empty CUs, so the slice count decides the time far more than the work
// does (784-300, 60000 samples, 65 tiles: 16 slices = 1040 work-groups 358 us, 15 slices 316 us, 23 slices =
// 1495 work-groups 303 us).  The count is the minimum of a model fitted to such sweeps: a K-tile step costs
// 0.925 us when 3 work-groups share a CU, 0.64 us with 2 and 0.335 us with 1 (last, partial round); every
// work-group adds 0.006 us for writing and folding its partial tile.
// b_kcont: the right operand is K-contiguous (the products): four work-groups per CU, 1.28 us per K-tile step then.
int pick_splits(int tiles, int K, bool b_kcont) {
    const int per_cu = b_kcont ? 4 : 3;
    const int kSlots = per_cu * 256;
    constexpr double kStep[5] = {0.0, 0.335, 0.64, 0.925, 1.28};
    const int smax = std::min(64, std::max(1, K / 256));
    int best = 1;
    double best_t = 0.0, one_t = 0.0;
    for (int s = 1; s <= smax; ++s) {
        const long long wgs = (long long)tiles * s;
        const int steps = cdiv(cdiv(K, s), 16);
        const int rounds = (int)(wgs / kSlots), rest = (int)(wgs % kSlots);
        const double t = steps * (rounds * kStep[per_cu] + kStep[std::min(per_cu, cdiv(rest, 256))]) + 0.006 * (double)wgs;
        if (s == 1) one_t = t;
        if (s == 1 || t < best_t) { best = s; best_t = t; }
    }
    // the model is good to a few percent: no slicing unless it promises more than that.  With the K-contiguous right
    // operand it gets the order of the candidates right but understates the gains (3072-1000-500-10, 2500 samples: 3
    // slices promised 2.5 %, measured 8 % on the launch; 2048-2000-2000-2000-100, 5000 samples: 2 slices, 2.3 % and 6.6 %),
    // so the bar is lower there.
    return one_t <= (b_kcont ? 1.015 : 1.03) * best_t ? 1 : best;
}

// Plan of the sums over samples  W_m = T^m^T [Z^{m-1}, 1]  for K samples.  grouped: all layers in
// one launch (product); otherwise one launch per layer (gradient).
// force_splits > 0: that many slices instead of the model's choice.
TnPlan plan_tn(const dn_ctx* c, int K, bool grouped, int only_layer, int force_splits = 0) {
    TnPlan pl;
    std::memset(&pl, 0, sizeof(pl));
    int tiles = 0;
    for (int m = 1; m <= c->L; ++m) {
        if (!grouped && m != only_layer) continue;
        tiles += cdiv(c->dims[m], 64) * cdiv(c->dims[m - 1] + 1, 64);
    }
    pl.splits = force_splits > 0 ? force_splits : pick_splits(tiles, K, grouped);
    pl.k_per_split = (int)round_up(cdiv(K, pl.splits), kBKmax);
    long long off = 0;
    for (int m = 1; m <= c->L; ++m) {
        pl.offset[m] = off;
        pl.floats[m] = (long long)pl.splits * tn_slice_floats(c, m);
        off += round_up(pl.floats[m], 64);
    }
    pl.total = off;
    return pl;
}

// The product's plan for s samples, with the slice count cut back to what the workspace's partial buffer holds.
// pick_splits is not monotone in K, so a smaller s than s_max can ask for more slices than the workspace was
// sized for (layout_workspace scans the counts up to s_max, this is the safety net); one slice always fits.
TnPlan plan_tn_product(const dn_ctx* c, int s) {
    TnPlan pl = plan_tn(c, s, true, 0);
    while (pl.total > c->tn_floats && pl.splits > 1) pl = plan_tn(c, s, true, 0, pl.splits - 1);
    return pl;
}

}  // namespace
