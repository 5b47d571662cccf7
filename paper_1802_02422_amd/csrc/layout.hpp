// Load-time kernels: the Eq. (7) constant table and the 16-byte aligned
// per-subregion record blocks the scan streams.
#pragma once
#include "util.hpp"

namespace ivf {

#ifndef IVF_BLK_ALIGN
#define IVF_BLK_ALIGN 16
#endif
constexpr int BLK_ALIGN = IVF_BLK_ALIGN;   // a 16-byte code is one aligned 128-bit load; tighter than the fetch granularity on purpose: measured fastest

// cst[r][l] = -alpha_r (1 - alpha_r) ||c_r - s_l||^2
__global__ __launch_bounds__(256) void cst_kernel(const float *__restrict__ alpha,
                                                  const float *__restrict__ cs_dist2, int L,
                                                  int64_t total, float *__restrict__ cst)
{
    int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= total) return;
    float a = alpha[i / L];
    cst[i] = -a * (1.f - a) * cs_dist2[i];
}

// size of each subregion's block in BLK_ALIGN-byte units
__global__ __launch_bounds__(256) void blk_size_kernel(const uint32_t *__restrict__ sub_offsets,
                                                       int64_t nsub, int M, uint32_t *__restrict__ sz)
{
    int64_t b = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (b >= nsub) return;
    uint32_t len = sub_offsets[b + 1] - sub_offsets[b];
    sz[b] = (len * (uint32_t)(M + 1) + BLK_ALIGN - 1) / BLK_ALIGN;
}

// copy subregion b's codes and constant bytes into its block; 16 lanes per subregion
__global__ __launch_bounds__(256) void repack_kernel(
    const uint32_t *__restrict__ sub_offsets, const uint32_t *__restrict__ blk_off, int64_t nsub,
    int M, const uint8_t *__restrict__ codes, const uint8_t *__restrict__ const_byte,
    uint8_t *__restrict__ blocks)
{
    int64_t b = ((int64_t)blockIdx.x * 256 + threadIdx.x) >> 4;
    int c_lane = threadIdx.x & 15;
    if (b >= nsub) return;
    uint32_t p0 = sub_offsets[b], len = sub_offsets[b + 1] - p0;
    uint8_t *blk = blocks + (uint64_t)blk_off[b] * BLK_ALIGN;
    for (uint32_t c = c_lane; c < len; c += 16) {
        const uint8_t *src = codes + ((uint64_t)p0 + c) * M;
        uint8_t *dst = blk + (uint64_t)c * M;
        if (M == 16) {
            *reinterpret_cast<uint4 *>(dst) = *reinterpret_cast<const uint4 *>(src);
        } else {
            *reinterpret_cast<uint2 *>(dst) = *reinterpret_cast<const uint2 *>(src);
        }
        blk[(uint64_t)len * M + c] = const_byte[(uint64_t)p0 + c];
    }
}

// one record per subregion with everything the pruning stage needs to describe it to the scan:
// block offset (BLK_ALIGN-byte units), first grouped position, length
__global__ __launch_bounds__(256) void sub_info_kernel(const uint32_t *__restrict__ sub_offsets,
                                                       const uint32_t *__restrict__ blk_off, int64_t nsub,
                                                       uint4 *__restrict__ info)
{
    int64_t b = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (b >= nsub) return;
    uint32_t p0 = sub_offsets[b];
    info[b] = make_uint4(blk_off[b], p0, sub_offsets[b + 1] - p0, 0u);
}

// plain streaming copy of n16 16-byte words (reference point for HBM counters and timings)
__global__ __launch_bounds__(256) void copy_bytes_kernel(const uint4 *__restrict__ src,
                                                         uint4 *__restrict__ dst, int64_t n16)
{
    int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const int64_t stride = (int64_t)gridDim.x * 256;
    for (; i < n16; i += stride) dst[i] = src[i];
}

}  // namespace ivf
