// Small device helpers shared by the kernels: order-preserving float keys,
// wavefront (64 lanes) and workgroup scans / reductions.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace ivf {

constexpr int WAVE = 64;
constexpr uint64_t EMPTY_KEY = ~0ull;

// fp32 -> uint32 such that a < b  <=>  key(a) < key(b) (for non-NaN values)
__device__ __forceinline__ uint32_t float_key(float f)
{
    uint32_t u = __float_as_uint(f);
    return u ^ ((u >> 31) ? 0xFFFFFFFFu : 0x80000000u);
}

__device__ __forceinline__ float key_float(uint32_t k)
{
    uint32_t u = k ^ ((k >> 31) ? 0x80000000u : 0xFFFFFFFFu);
    return __uint_as_float(u);
}

// LDS traffic between lanes of one wavefront: keep the compiler from moving
// LDS accesses across this point (the hardware executes a wave's LDS
// instructions in order).
__device__ __forceinline__ void wave_sync()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// DPP move with 0 for lanes that have no source (shifted out of their row of 16,
// or in a row excluded by ROW_MASK).
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ uint32_t dpp_or_zero(uint32_t v)
{
    return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, CTRL, ROW_MASK, 0xf, false);
}

// Inclusive prefix sum over the 64 lanes in 6 DPP steps, no LDS: row_shr 1/2/4/8 scan each row
// of 16, row_bcast15 carries rows 0,2 into rows 1,3, row_bcast31 carries lane 31 into rows 2,3.
__device__ __forceinline__ uint32_t wave_inclusive_scan(uint32_t v)
{
    v += dpp_or_zero<0x111, 0xf>(v);
    v += dpp_or_zero<0x112, 0xf>(v);
    v += dpp_or_zero<0x114, 0xf>(v);
    v += dpp_or_zero<0x118, 0xf>(v);
    v += dpp_or_zero<0x142, 0xa>(v);
    v += dpp_or_zero<0x143, 0xc>(v);
    return v;
}

__device__ __forceinline__ float wave_sum(float v)
{
#pragma unroll
    for (int o = WAVE / 2; o > 0; o >>= 1) v += __shfl_xor(v, o, WAVE);
    return v;
}

__device__ __forceinline__ double wave_sum(double v)
{
#pragma unroll
    for (int o = WAVE / 2; o > 0; o >>= 1) v += __shfl_xor(v, o, WAVE);
    return v;
}

// argmin over the wave of (value, index) pairs, lowest index on equal values;
// every lane receives the winner.
__device__ __forceinline__ void wave_argmin(float &v, int &idx)
{
#pragma unroll
    for (int o = WAVE / 2; o > 0; o >>= 1) {
        float ov = __shfl_xor(v, o, WAVE);
        int oi = __shfl_xor(idx, o, WAVE);
        if (ov < v || (ov == v && oi < idx)) { v = ov; idx = oi; }
    }
}

__device__ __forceinline__ void wave_argmin(double &v, int &idx)
{
#pragma unroll
    for (int o = WAVE / 2; o > 0; o >>= 1) {
        double ov = __shfl_xor(v, o, WAVE);
        int oi = __shfl_xor(idx, o, WAVE);
        if (ov < v || (ov == v && oi < idx)) { v = ov; idx = oi; }
    }
}

// Exclusive scan of one uint32 per thread over a workgroup of BLOCK threads
// (BLOCK a multiple of 64).  sh must hold BLOCK/64 words of LDS.  Returns the
// exclusive prefix; total receives the workgroup sum.  Contains barriers.
template <int BLOCK>
__device__ __forceinline__ uint32_t block_exclusive_scan(uint32_t v, uint32_t *sh, uint32_t &total)
{
    constexpr int NW = BLOCK / WAVE;
    const int lane = threadIdx.x & (WAVE - 1), w = threadIdx.x / WAVE;
    uint32_t inc = wave_inclusive_scan(v);
    if (lane == WAVE - 1) sh[w] = inc;
    __syncthreads();
    uint32_t before = 0, tot = 0;
#pragma unroll
    for (int i = 0; i < NW; ++i) {
        uint32_t s = sh[i];
        if (i < w) before += s;
        tot += s;
    }
    __syncthreads();
    total = tot;
    return before + inc - v;
}

}  // namespace ivf
