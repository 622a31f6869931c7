// Limits shared by the kernels and the host code, and the wave / work-group reductions.
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

// Four floats of a stored block, 16-byte aligned, fetched as a streaming (non-temporal) load: the blocks are read
// once per product and are far larger than the caches, and a read that does not allocate there runs at 6.9-7.1 TB/s
// on MI355X where a plain one reaches 6.1-6.3 (16 GB, float4 per lane, 2048 work-groups).  Used by the kernels that
// stream blocks from HBM (teams of work-groups, two-pass kernels); the register-strip kernels serve narrow outputs,
// whose blocks mostly fit the memory-side cache between products, and keep plain loads (measured: no gain there).
typedef float dn_f32x4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ float4 load_stream4(const float* p) {
    const dn_f32x4 v = __builtin_nontemporal_load(reinterpret_cast<const dn_f32x4*>(p));
    return make_float4(v[0], v[1], v[2], v[3]);
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

}  // namespace dn
