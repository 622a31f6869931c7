// Single pass over the stored blocks by teams of work-groups sharing a sample (wide outputs, n_L > 16, and narrow
// ones whose hidden layers exceed the register-strip kernel).
#pragma once
#include "dn_common.h"
#include "dn_kernels_stream.h"

namespace dn {

// ---------------------------------------------------------------------------------------------
// The two products of Section 4.2 need every element of P^m_i twice, and r_i = J_i v must be complete
// before the transposed product can start.  One sample's blocks (n_L x sum n_m floats) exceed what one
// work-group can hold, so a TEAM of work-groups shares a sample: work-group cs of a team owns a column
// slice (up to 1024 columns of one layer, 4 KB of every row) and walks down the rows of the sample in bands
// of at most H rows, which it keeps in registers:
//   A. partial sums r_cs[u] = sum_{j in slice} P[u][j] q[j] for the band's rows  ->  exchange words
//   B. EVERY work-group reads the partial sums of all slices that share the sum and adds them in the same
//      fixed order (so all hold the same bits), adds q^L (full mode) and doubles (B = 2I)
//   C. t[j] += sum_{u in band} P[u][j] 2r[u] from the registers; after the last band of the sample t goes
//      to memory.
// Each stored element is thus read from HBM once per product, in runs of 4 KB, and one exchange (a store
// and a poll, no second hop through a folding work-group) separates the two uses.
// Which partial sums share a sum: all slices (full matrix), the slices of the same layer (per-layer
// blocks, Section 4.1), or the slices of the same output group of the same layer, once per input group
// (partitions of a split structure, Section 3.1: GA > 1 vectors q^{m,a} per slice).
// The kernel is persistent: the host sizes the grid (teams x slices) to be resident all at once, and team
// t walks over samples t, t + teams, ...
// Exchange between work-groups: every float travels in a 64-bit word together with a sequence number
// (base + bands done + 1, never 0), written and read with single device-scope atomic accesses.  Those
// go through to memory, past the XCD-private L2s, so no cache write-back or invalidation is needed, and a
// reader simply polls the word until it carries the expected number.  Two sets of words are used
// alternately: a work-group writes set k & 1 for its k-th band after it has read all words of band k-1,
// which exist only after every work-group of the team has finished reading band k-2, the previous user of
// that set.
// The base lives in device memory: every work-group reads it when it starts and the last one to finish moves it on
// by the launch's count, so a launch that is replayed from a captured graph gets fresh numbers each time (numbers
// baked into the launch arguments would repeat, and a word left by the previous replay could then pass for this
// one's).  When the numbers are about to wrap that work-group also clears the exchange words.
// Every wait is bounded: after spin_limit polls a thread raises the error word and its work-group leaves;
// so does every work-group that sees the error word raised.  The host then runs the two-pass kernels on
// the same product (they are enqueued behind this kernel and do nothing unless the word is raised).
#define DN_MAX_BAND_SLICES 48

struct BandSlice {
    int m;          // layer
    int j0;         // first column the slice loads (multiple of 4)
    int lo, hi;     // its own columns [lo, hi), j0 <= lo < hi <= j0 + 1024
    int c_lo, c_hi; // slices whose partial sums are added together with this one's
};

struct BandArgs {
    int L, s, nL;
    int mode;                            // 0 full, 1 per-layer, 2 partitions
    long long ld[DN_MAX_LAYERS + 1];
    const float* P[DN_MAX_LAYERS + 1];   // [s][nL][ld[m]]
    const float* Q[DN_MAX_LAYERS + 1];   // [ga][s][ld[m]] (ga = 1 outside partition mode)
    float* T[DN_MAX_LAYERS + 1];         // [ga][s][ld[m]]
    int ga[DN_MAX_LAYERS + 1];           // input groups of layer m
    int ncs, teams, nrs, rps;            // slices, teams, bands per sample, rows per band (<= H)
    BandSlice sl[DN_MAX_BAND_SLICES];
    unsigned* seq;                       // seq[0]: sequence numbers handed out so far (the launch's base), seq[1]: work-groups
                                         // of this launch that have finished
    unsigned per_launch;                 // sequence numbers this launch uses: bands per team + 1
    long long exch_words;                // size of the exchange buffer (cleared when the numbers wrap)
    unsigned long long* part;            // [teams][2][ncs][GA][32]
    unsigned* error;                     // one word, nonzero after a wait ran out
    unsigned spin_limit;
    unsigned long long* clk;             // nullable: per work-group, shader-clock cycles spent in each phase (see below)
};

// Phase clocks (diagnostic, template parameter CLK; the clocked variant needs BandArgs::clk): thread 0 of every work-group adds up the shader-clock
// cycles between its band's first load and the barrier behind the partial sums (loading), from there to the barrier
// behind the exchange (waiting for the slowest work-group of the team, plus the round trip through memory), and
// from there to the end of the band (transposed product), and leaves the three sums and its band count in clk[4 b ..].
#define DN_BAND_CLK(k) do { if (CLK && tid == 0) clk_t[k] = __builtin_readcyclecounter(); } while (0)

__device__ __forceinline__ unsigned long long ll_pack(float v, unsigned seq) {
    return ((unsigned long long)seq << 32) | (unsigned long long)__builtin_bit_cast(unsigned, v);
}
__device__ __forceinline__ void ll_store(unsigned long long* p, float v, unsigned seq) {
    __hip_atomic_store(p, ll_pack(v, seq), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ unsigned long long ll_load(const unsigned long long* p) {
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// acc[a] += the floats in base[a * 32], a < ga, once all of them carry `seq`.  Returns false if the wait
// ran out (error word raised).
template <int GA>
__device__ __forceinline__ bool ll_take(const unsigned long long* base, int ga, unsigned seq, unsigned* error,
                                        unsigned spin_limit, float (&acc)[GA]) {
    unsigned long long w[GA];
    bool got = false;
    for (unsigned spins = 0; spins < spin_limit; ++spins) {
        bool all = true;
#pragma unroll
        for (int a = 0; a < GA; ++a) {
            w[a] = a < ga ? ll_load(base + a * 32) : ((unsigned long long)seq << 32);
            all = all && ((unsigned)(w[a] >> 32) == seq);
        }
        if (all) { got = true; break; }
        if ((spins & 63u) == 63u && __hip_atomic_load(error, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0u) break;
        __builtin_amdgcn_s_sleep(2);
    }
    if (!got) {
        __hip_atomic_store(error, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        return false;
    }
#pragma unroll
    for (int a = 0; a < GA; ++a) acc[a] += __builtin_bit_cast(float, (unsigned)(w[a] & 0xffffffffull));
    return true;
}

// H rows per band, all in registers; thread (wave w, lane) owns columns j0 + 256 w + 4 lane .. + 3 of every row.
template <int H, int GA, int WAVES_PER_SIMD, bool CLK = false>
__global__ __launch_bounds__(256, WAVES_PER_SIMD) void jv_jtv_band_kernel(const BandArgs ba) {
    static_assert(H <= 32, "a band's rows are exchanged in vectors of 32 words");
    __shared__ float wpart[4][GA][32];     // per-wave partial r of this slice
    __shared__ float fold[8][GA][32];
    __shared__ float r2[GA][32];           // 2 r of the band's rows
    __shared__ int flag;

    const int team = blockIdx.x / ba.ncs, cs = blockIdx.x - team * ba.ncs;
    const int tid = threadIdx.x, lane = tid & 63;
    // the wave index as a scalar: row addresses are then scalar bases plus one per-lane column offset
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const BandSlice sl = ba.sl[cs];
    const int m = sl.m;
    const int j = sl.j0 + wave * 256 + 4 * lane;
    const bool live = j + 3 >= sl.lo && j < sl.hi;                 // at least one own column
    const bool edge = live && (j < sl.lo || j + 3 >= sl.hi);       // some of the four are not this slice's
    const long long ldm = ba.ld[m];
    const int nL = ba.nL, L = ba.L;
    const int ga = GA > 1 ? ba.ga[m] : 1;
    const long long qstride = (long long)ba.s * ldm;               // between the Q / T of successive input groups
    unsigned long long* part_team = ba.part + (long long)team * 2 * ba.ncs * GA * 32;

    // a wait that ran out in an earlier launch: do nothing (the two-pass kernels behind this one do the work)
    if (tid == 0) flag = __hip_atomic_load(ba.error, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == 0u ? 1 : 0;
    __syncthreads();
    if (!flag) return;
    const unsigned seq_base = ba.seq[0];      // written by the previous launch's last work-group (or the clear kernel)

    // columns that are padding or belong to a neighbouring slice stay out of the sums
    auto mask = [&](float4& x) {
        if (edge) {
            if (j + 0 < sl.lo || j + 0 >= sl.hi) x.x = 0.f;
            if (j + 1 < sl.lo || j + 1 >= sl.hi) x.y = 0.f;
            if (j + 2 < sl.lo || j + 2 >= sl.hi) x.z = 0.f;
            if (j + 3 < sl.lo || j + 3 >= sl.hi) x.w = 0.f;
        }
    };
    const int ul = tid & 31, sub = tid >> 5;

    __shared__ unsigned long long clk_sum[3], clk_t[3];
    if (tid < 3) clk_sum[tid] = 0ull;     // (the barrier below the error check orders this before any use)
    unsigned done = 0;        // bands this team has finished
    for (int i = team; i < ba.s; i += ba.teams) {
        float4 q4[GA], tacc[GA];
#pragma unroll
        for (int a = 0; a < GA; ++a) {
            q4[a] = make_float4(0.f, 0.f, 0.f, 0.f);
            tacc[a] = make_float4(0.f, 0.f, 0.f, 0.f);
            if (live && a < ga) q4[a] = *reinterpret_cast<const float4*>(ba.Q[m] + a * qstride + (long long)i * ldm + j);
        }
        for (int rs = 0; rs < ba.nrs; ++rs, ++done) {
            const unsigned seq = seq_base + done + 1u;
            unsigned long long* part_cur = part_team + (long long)(done & 1u) * ba.ncs * GA * 32;
            const int u0 = rs * ba.rps;
            const int nrow = min(ba.rps, nL - u0);
            // ---- A: load the band, partial J v ------------------------------------------------
            DN_BAND_CLK(0);
            const float* __restrict__ prow = ba.P[m] + ((long long)i * nL + u0) * ldm + j;
            float4 p[H];
#pragma unroll
            for (int k = 0; k < H; ++k) {
                p[k] = make_float4(0.f, 0.f, 0.f, 0.f);
                if (live && k < nrow) p[k] = load_stream4(prow + (long long)k * ldm);
            }
            // q^L of the band's rows (full mode) is fetched now, not after the wait
            float qL = 0.f;
            if (ba.mode != 2 && tid < nrow) qL = ba.Q[L][(long long)i * ba.ld[L] + u0 + tid];
            if (GA > 1 && ba.mode == 2 && cs == 0 && tid < nrow) {
                // output layer of a split structure: the identity block, t^{L,a} = 2 q^{L,a} for every input group
                for (int a = 0; a < ba.ga[L]; ++a) {
                    const long long e = ((long long)a * ba.s + i) * ba.ld[L] + u0 + tid;
                    ba.T[L][e] = 2.0f * ba.Q[L][e];
                }
            }
            if (rs == 0) {
#pragma unroll
                for (int a = 0; a < GA; ++a) mask(q4[a]);
            }
#pragma unroll
            for (int k = 0; k < H; ++k) {
                mask(p[k]);
#pragma unroll
                for (int a = 0; a < GA; ++a) {
                    if (a < ga) {
                        float x = p[k].x * q4[a].x + p[k].y * q4[a].y + p[k].z * q4[a].z + p[k].w * q4[a].w;
                        x = wave_sum_to_lane63(x);
                        if (lane == 63) wpart[wave][a][k] = x;      // rows past the band get zeros (p was zero)
                    }
                }
            }
            __syncthreads();
            DN_BAND_CLK(1);
            if (ul < H && sub < ga)
                ll_store(&part_cur[((long long)cs * GA + sub) * 32 + ul],
                         (wpart[0][sub][ul] + wpart[1][sub][ul]) + (wpart[2][sub][ul] + wpart[3][sub][ul]), seq);

            // ---- B: every work-group adds the partial sums of the slices that share this sum ---------
            bool ok = true;
            {
                float acc[GA];
#pragma unroll
                for (int a = 0; a < GA; ++a) acc[a] = 0.f;
                if (ul < H)
                    for (int c = sl.c_lo + sub; c < sl.c_hi && ok; c += 8)
                        ok = ll_take<GA>(part_cur + (long long)c * GA * 32 + ul, ga, seq, ba.error, ba.spin_limit, acc);
#pragma unroll
                for (int a = 0; a < GA; ++a) fold[sub][a][ul] = acc[a];
            }
            if (!__syncthreads_and(ok ? 1 : 0)) return;
            DN_BAND_CLK(2);
            if (ul < H && sub < ga) {
                const int a = sub;
                float r = ((fold[0][a][ul] + fold[1][a][ul]) + (fold[2][a][ul] + fold[3][a][ul])) +
                          ((fold[4][a][ul] + fold[5][a][ul]) + (fold[6][a][ul] + fold[7][a][ul]));
                if (ul < nrow) {
                    if (ba.mode == 0) {
                        r = 2.0f * (r + qL);
                        if (cs == 0) ba.T[L][(long long)i * ba.ld[L] + u0 + ul] = r;          // t^L = 2 r
                    } else {
                        r = 2.0f * r;
                        if (ba.mode == 1 && cs == 0) ba.T[L][(long long)i * ba.ld[L] + u0 + ul] = 2.0f * qL;
                    }
                } else {
                    r = 0.f;
                }
                r2[a][ul] = r;
            }
            __syncthreads();
            // ---- C: transposed product from the registers --------------------------------------
#pragma unroll
            for (int k = 0; k < H; ++k) {
#pragma unroll
                for (int a = 0; a < GA; ++a) {
                    if (a < ga) {
                        const float w = r2[a][k];             // zero for rows past the band
                        tacc[a].x += p[k].x * w; tacc[a].y += p[k].y * w; tacc[a].z += p[k].z * w; tacc[a].w += p[k].w * w;
                    }
                }
            }
            if (CLK && tid == 0) {
                const unsigned long long c3 = __builtin_readcyclecounter();
                clk_sum[0] += clk_t[1] - clk_t[0]; clk_sum[1] += clk_t[2] - clk_t[1]; clk_sum[2] += c3 - clk_t[2];
            }
        }
        if (live) {
#pragma unroll
            for (int a = 0; a < GA; ++a) {
                if (a < ga) {
                    float* dst = ba.T[m] + a * qstride + (long long)i * ldm + j;
                    if (!edge) {
                        *reinterpret_cast<float4*>(dst) = tacc[a];
                    } else {
                        if (j + 0 >= sl.lo && j + 0 < sl.hi) dst[0] = tacc[a].x;
                        if (j + 1 >= sl.lo && j + 1 < sl.hi) dst[1] = tacc[a].y;
                        if (j + 2 >= sl.lo && j + 2 < sl.hi) dst[2] = tacc[a].z;
                        if (j + 3 >= sl.lo && j + 3 < sl.hi) dst[3] = tacc[a].w;
                    }
                }
            }
        }
    }
    // the last work-group to finish moves the base on (all others have read it long ago)
    if (tid == 0) flag = __hip_atomic_fetch_add(&ba.seq[1], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == gridDim.x - 1u ? 1 : 0;
    __syncthreads();
    if (flag) {
        unsigned next = seq_base + ba.per_launch;
        if (next > 0x7fff0000u) {
            for (long long e = tid; e < ba.exch_words; e += 256) ba.part[e] = 0ull;
            next = 0u;
        }
        if (tid == 0) {
            ba.seq[0] = next;
            ba.seq[1] = 0u;
        }
    }
    if (CLK && tid == 0 && ba.clk) {
        ba.clk[blockIdx.x * 4 + 0] = clk_sum[0]; ba.clk[blockIdx.x * 4 + 1] = clk_sum[1];
        ba.clk[blockIdx.x * 4 + 2] = clk_sum[2]; ba.clk[blockIdx.x * 4 + 3] = done;
    }
}

// exchange words to zero (sequence number 0 = nothing written) once after the workspace is bound
__global__ void band_clear_kernel(unsigned long long* words, long long n, unsigned* error, unsigned* seq) {
    for (long long e = (long long)blockIdx.x * blockDim.x + threadIdx.x; e < n; e += (long long)gridDim.x * blockDim.x)
        words[e] = 0ull;
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        *error = 0u;
        seq[0] = 0u;
        seq[1] = 0u;
    }
}

}  // namespace dn
