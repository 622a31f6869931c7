// Single pass over the stored blocks for wide outputs: teams of work-groups sharing a sample.
#pragma once
#include "dn_common.h"
#include "dn_kernels_stream.h"

namespace dn {

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

}  // namespace dn
