// Stages 5-6: the asymmetric-distance scan of the kept subregions with
// per-wavefront top-k pools (Eq. (6)), and the final k-select.
//
// Record layout (built at load time): subregion b owns a 64-byte aligned block
// at byte offset 64*blk_off[b] holding len*M code bytes followed by len
// constant-term bytes, so one subregion is one contiguous HBM run.
#pragma once
#include "query.hpp"

namespace ivf {

constexpr int SCAN_BLOCK = 256;
constexpr int SCAN_WAVES = SCAN_BLOCK / WAVE;

__host__ __device__ inline int pool_capacity(int k)
{
    int cap = 128;
    while (cap < 2 * k) cap <<= 1;
    return cap;
}

template <int M> struct CodeWord;
template <> struct CodeWord<16> { typedef uint4 type; };
template <> struct CodeWord<8> { typedef uint2 type; };

template <int M>
__device__ __forceinline__ float adc_sum(const typename CodeWord<M>::type &c, const float *T, float acc);

template <>
__device__ __forceinline__ float adc_sum<16>(const uint4 &c, const float *T, float acc)
{
    const uint32_t w[4] = {c.x, c.y, c.z, c.w};
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int b = 0; b < 4; ++b) acc += T[(4 * i + b) * 256 + ((w[i] >> (8 * b)) & 255u)];
    return acc;
}

template <>
__device__ __forceinline__ float adc_sum<8>(const uint2 &c, const float *T, float acc)
{
    const uint32_t w[2] = {c.x, c.y};
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int b = 0; b < 4; ++b) acc += T[(4 * i + b) * 256 + ((w[i] >> (8 * b)) & 255u)];
    return acc;
}

// Sort the wave's pool, keep its k best, return the new admission threshold.
__device__ __forceinline__ float wave_pool_compact(uint64_t *pool, int cap, int &pool_n, int k)
{
    const int lane = threadIdx.x & (WAVE - 1);
    for (int i = pool_n + lane; i < cap; i += WAVE) pool[i] = EMPTY_KEY;
    wave_bitonic_sort(pool, cap);
    if (pool_n > k) pool_n = k;
    float theta = INFINITY;
    if (pool_n == k) theta = key_float((uint32_t)(pool[k - 1] >> 32));
    return theta;
}

// Grid: nq * nsplit workgroups; workgroup (q, split) scans an equal share of
// the query's S descriptors.  A group of 16 lanes walks one subregion, one
// record per lane per step (a 16-byte code load at M = 16), looks the M bytes
// up in the query's table held in LDS, adds the subregion base and the
// dequantised constant byte, and offers the estimate to its wavefront's pool.
// Output: per (q, split, wave) the k best keys (distance, id), ascending,
// padded with EMPTY_KEY.
template <int M>
__global__ __launch_bounds__(SCAN_BLOCK) void scan_kernel(
    const uint8_t *__restrict__ blocks, const int32_t *__restrict__ ids,
    const float *__restrict__ const_table, const SubDesc *__restrict__ desc, int S,
    const float *__restrict__ lut, int k, int nsplit, uint64_t *__restrict__ partial)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    float *T = reinterpret_cast<float *>(smem);                 // M*256
    float *nt = T + M * 256;                                    // 256
    uint64_t *pools = reinterpret_cast<uint64_t *>(nt + 256);   // SCAN_WAVES * cap
    typedef typename CodeWord<M>::type code_t;

    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int64_t q = blockIdx.x / nsplit;
    const int split = blockIdx.x % nsplit;
    const int cap = pool_capacity(k);
    uint64_t *pool = pools + wave * cap;

    {
        const float4 *src = reinterpret_cast<const float4 *>(lut + q * (int64_t)(M * 256));
        float4 *dst = reinterpret_cast<float4 *>(T);
        for (int i = tid; i < M * 64; i += SCAN_BLOCK) dst[i] = src[i];
        nt[tid] = const_table[tid];
    }
    __syncthreads();

    const int d_begin = (int)(((int64_t)S * split) / nsplit);
    const int d_end = (int)(((int64_t)S * (split + 1)) / nsplit);
    const SubDesc *qd = desc + q * S;
    const int g = lane >> 4, c_lane = lane & 15;

    int pool_n = 0;
    float theta = INFINITY;

    for (int d0 = d_begin + wave * 4; d0 < d_end; d0 += SCAN_WAVES * 4) {
        const int d = d0 + g;
        SubDesc sd;
        sd.blk = 0; sd.pos0 = 0; sd.len = 0; sd.base = 0.f;
        if (d < d_end) sd = qd[d];
        uint32_t maxlen = sd.len;
#pragma unroll
        for (int o = 32; o >= 16; o >>= 1) {
            uint32_t t = __shfl_xor(maxlen, o, WAVE);
            maxlen = t > maxlen ? t : maxlen;
        }
        const uint8_t *blk = blocks + (uint64_t)sd.blk * 64u;
        for (uint32_t c0 = 0; c0 < maxlen; c0 += 16) {
            const uint32_t c = c0 + c_lane;
            const bool active = c < sd.len;
            float dist = INFINITY;
            if (active) {
                code_t code = *reinterpret_cast<const code_t *>(blk + (uint64_t)c * M);
                uint32_t cb = blk[(uint64_t)sd.len * M + c];
                dist = adc_sum<M>(code, T, sd.base + nt[cb]);
            }
            const bool pass = active && dist <= theta;
            const uint64_t mask = __ballot(pass);
            if (mask) {
                if (pass) {
                    int slot = pool_n + __popcll(mask & ((1ull << lane) - 1ull));
                    pool[slot] = dist_id_key(dist, ids[sd.pos0 + c]);
                }
                pool_n += __popcll(mask);
                if (pool_n > cap - WAVE) theta = wave_pool_compact(pool, cap, pool_n, k);
            }
        }
    }
    wave_pool_compact(pool, cap, pool_n, k);
    uint64_t *out = partial + ((q * nsplit + split) * SCAN_WAVES + wave) * (int64_t)k;
    for (int i = lane; i < k; i += WAVE) out[i] = i < pool_n ? pool[i] : EMPTY_KEY;
}

// Final k-select: sort the n_lists * k partial keys of a query and write the k
// best as (id, distance); empty slots become (-1, +inf).
template <int BLOCK>
__global__ __launch_bounds__(BLOCK) void merge_kernel(const uint64_t *__restrict__ partial, int n_in,
                                                      int n_pow2, int k, int32_t *__restrict__ out_ids,
                                                      float *__restrict__ out_dists)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    uint64_t *a = reinterpret_cast<uint64_t *>(smem);
    const int64_t q = blockIdx.x;
    for (int i = threadIdx.x; i < n_pow2; i += BLOCK) a[i] = i < n_in ? partial[q * n_in + i] : EMPTY_KEY;
    block_bitonic_sort<BLOCK>(a, n_pow2);
    for (int i = threadIdx.x; i < k; i += BLOCK) {
        uint64_t key = i < n_pow2 ? a[i] : EMPTY_KEY;
        bool empty = key == EMPTY_KEY;
        out_ids[q * k + i] = empty ? -1 : (int32_t)(uint32_t)key;
        out_dists[q * k + i] = empty ? INFINITY : key_float((uint32_t)(key >> 32));
    }
}

}  // namespace ivf
