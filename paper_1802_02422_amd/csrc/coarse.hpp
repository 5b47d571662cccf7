// Stage 1: squared distances from a tile of queries to all K centroids as an
// fp32 MFMA GEMM (||q||^2 - 2<q,c> + ||c||^2), and the exact per-query
// selection of the nprobe closest regions (exhaustive assignment, Section 3.1).
#pragma once
#include "select.hpp"

namespace ivf {

typedef float floatx16 __attribute__((ext_vector_type(16)));

// ||row||^2 of an [n][D] fp32 matrix, one wavefront per row.
__global__ __launch_bounds__(256) void row_norm_kernel(const float *__restrict__ X, int64_t n,
                                                       int D, float *__restrict__ out)
{
    int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    int lane = threadIdx.x & 63;
    if (row >= n) return;
    float s = 0.f;
    for (int i = lane; i < D; i += WAVE) {
        float v = X[row * D + i];
        s = fmaf(v, v, s);
    }
    s = wave_sum(s);
    if (lane == 0) out[row] = s;
}

constexpr int GT = 128;        // tile: GT queries x GT centroids per workgroup
constexpr int GKC = 32;        // dimensions staged per step
constexpr int GLD = GKC + 4;   // LDS row stride in floats (keeps 16-byte alignment, spreads banks)

// One 128x128 tile of <Q[q], C[j]> per workgroup of 4 wavefronts; each
// wavefront owns a 64x64 quadrant as 2x2 v_mfma_f32_32x32x2f32 accumulators.
// Within each 16-dim half of a 32-dim stage lane half h feeds dims [8h, 8h+8) to
// both operands, so one ds_read_b128 serves four MFMA steps (the order of the
// k-summation is free; all variants of the kernel use the same one, so a query's
// distances do not depend on the batch it arrives in).  The centroids are the MFMA's row operand and the queries its column
// operand: in acc[i][j], lane l holds query (column) wq + 32i + l%32 and element
// v is centroid (row) wc + 32j + 8*(v/4) + 4*(l/32) + v%4, i.e. four groups of
// four consecutive centroids, which the epilogues store as 128-bit words and
// reduce without leaving the lane.
__device__ __forceinline__ void gemm_tile(const float *__restrict__ Q, int64_t nq, int64_t q0,
                                          const float *__restrict__ C, int64_t K, int64_t c0, int D,
                                          float *As, float *Bs, floatx16 (&acc)[2][2])
{
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int wq = (wave >> 1) * 64, wc = (wave & 1) * 64;
    const int l32 = lane & 31, h = lane >> 5;
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    // the global loads of stage s+1 are issued before the MFMA block of stage s and
    // land in registers while it runs
    float4 pa[4], pb[4];
    auto fetch = [&](int k0) {
#pragma unroll
        for (int it = 0; it < 4; ++it) {
            int idx = tid + it * 256;
            int row = idx >> 3, c4 = (idx & 7) * 4;
            // rows past the end are clamped to the last row (their products are never stored), columns
            // past D read column 0 and are zeroed: every load is unconditional
            const bool kv = k0 + c4 < D;
            const int64_t qrow = q0 + row < nq ? q0 + row : nq - 1, crow = c0 + row < K ? c0 + row : K - 1;
            const int col = kv ? k0 + c4 : 0;
            pa[it] = *reinterpret_cast<const float4 *>(Q + qrow * D + col);
            pb[it] = *reinterpret_cast<const float4 *>(C + crow * D + col);
            if (!kv) {
                pa[it] = make_float4(0.f, 0.f, 0.f, 0.f);
                pb[it] = pa[it];
            }
        }
    };
    fetch(0);
    for (int k0 = 0; k0 < D; k0 += GKC) {
#pragma unroll
        for (int it = 0; it < 4; ++it) {
            int idx = tid + it * 256;
            int row = idx >> 3, c4 = (idx & 7) * 4;
            *reinterpret_cast<float4 *>(&As[row * GLD + c4]) = pa[it];
            *reinterpret_cast<float4 *>(&Bs[row * GLD + c4]) = pb[it];
        }
        __syncthreads();
        if (k0 + GKC < D) fetch(k0 + GKC);
#pragma unroll
        for (int s4 = 0; s4 < 4; ++s4) {
            float4 a[2], b[2];
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                // same k order as the DMA variant: sub-stages of 16 dims, lane half h feeds [8h, 8h+8)
                const int kc = (s4 >> 1) * 16 + h * 8 + (s4 & 1) * 4;
                a[i] = *reinterpret_cast<const float4 *>(&As[(wq + i * 32 + l32) * GLD + kc]);
                b[i] = *reinterpret_cast<const float4 *>(&Bs[(wc + i * 32 + l32) * GLD + kc]);
            }
            // the four accumulators are independent: cycle through them so that no MFMA
            // waits for the one issued just before it
#pragma unroll
            for (int e = 0; e < 4; ++e)
#pragma unroll
                for (int i = 0; i < 2; ++i)
#pragma unroll
                    for (int j = 0; j < 2; ++j) {
                        const float av = e == 0 ? a[i].x : e == 1 ? a[i].y : e == 2 ? a[i].z : a[i].w;
                        const float bv = e == 0 ? b[j].x : e == 1 ? b[j].y : e == 2 ? b[j].z : b[j].w;
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(bv, av, acc[i][j], 0, 0, 0);
                    }
        }
        __syncthreads();
    }
}

constexpr int BMW = 64;   // centroids per block minimum
constexpr int N_XCD = 8;  // workgroups are dealt round-robin to the 8 XCDs, each with its own L2

// Tile of workgroup b: XCD x = b % 8 owns the query tiles x, x+8, ... (a few hundred KB that
// stay in its L2) and sweeps the centroid tiles in order, so every XCD streams the centroid
// matrix once and the eight of them work on the same centroid tile at about the same time.
__device__ __forceinline__ bool tile_of_block(int64_t b, int tiles_q, int64_t &q0, int64_t &c0)
{
    const int tq_per = (tiles_q + N_XCD - 1) / N_XCD;
    const int xcd = (int)(b % N_XCD);
    const int64_t local = b / N_XCD;
    const int tq = (int)(local % tq_per) * N_XCD + xcd;
    q0 = (int64_t)tq * GT;
    c0 = (local / tq_per) * GT;
    return tq < tiles_q;
}

// Dt[q][j] = max(0, qn[q] + cn[j] - 2 <Q[q], C[j]>), and bm[q][b] = the minimum
// of Dt[q][64b .. 64b+63] (each wavefront's 64-centroid quadrant gives one block
// minimum per query).  The grid has 8 * ceil(tiles_q / 8) * tiles_c workgroups.
// The same tile product with asynchronous operand staging, for D a multiple of 16: stages of
// 16 dims, operands copied global -> LDS by global_load_lds_dwordx4 (no registers, no ds_write),
// two LDS buffers so that the copy of stage s+1 runs under the MFMA block of stage s with one
// barrier per stage.  A direct-to-LDS load puts lane i's 16 bytes at base + 16 i, so the layout
// is unpadded rows of four float4; bank conflicts of the operand reads are avoided by storing
// float4 f of row r in slot f ^ ((r >> 2) & 3) (each lane simply fetches the float4 that belongs
// to its slot).  Lane half h feeds dims [8h, 8h+8) of the stage.  buf holds 2 x (128 + 128) rows
// x 16 floats.
constexpr int DK = 16;                       // dims per stage
constexpr int DBUF = 2 * GT * DK;            // floats per buffer (A rows then B rows)

__device__ __forceinline__ void gemm_tile_dma(const float *__restrict__ Q, int64_t nq, int64_t q0,
                                              const float *__restrict__ C, int64_t K, int64_t c0, int D,
                                              float *buf, floatx16 (&acc)[2][2])
{
    typedef const __attribute__((address_space(1))) void *gptr_t;
    typedef __attribute__((address_space(3))) void *lptr_t;
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int wq = (wave >> 1) * 64, wc = (wave & 1) * 64;
    const int l32 = lane & 31, h = lane >> 5;
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    // this wave's four copy instructions per stage: blocks of 16 rows; blocks 0-7 are query rows,
    // 8-15 centroid rows.  Rows past the end are clamped (their products are never stored).
    const float *src[4];
#pragma unroll
    for (int n = 0; n < 4; ++n) {
        const int blk = wave * 4 + n;
        const int r = (blk & 7) * 16 + (lane >> 2);                    // row inside the operand tile
        const int f = (lane & 3) ^ ((r >> 2) & 3);                     // float4 of the row this slot holds
        if (blk < 8) {
            const int64_t row = q0 + r < nq ? q0 + r : nq - 1;
            src[n] = Q + row * D + f * 4;
        } else {
            const int64_t row = c0 + r < K ? c0 + r : K - 1;
            src[n] = C + row * D + f * 4;
        }
    }
    auto issue = [&](int k0, float *dst) {
#pragma unroll
        for (int n = 0; n < 4; ++n)
            __builtin_amdgcn_global_load_lds((gptr_t)(src[n] + k0), (lptr_t)(dst + (wave * 4 + n) * 256), 16, 0, 0);
    };
    const int stages = D / DK;
    issue(0, buf);
    for (int s = 0; s < stages; ++s) {
        __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0): this wave's copies of stage s have landed
        __syncthreads();                      // ... and everyone's; all waves are done with the other buffer
        if (s + 1 < stages) issue((s + 1) * DK, buf + ((s + 1) & 1) * DBUF);
        const float *As = buf + (s & 1) * DBUF, *Bs = As + GT * DK;
#pragma unroll
        for (int s4 = 0; s4 < 2; ++s4) {
            float4 a[2], b[2];
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                const int ra = wq + i * 32 + l32, rb = wc + i * 32 + l32;
                a[i] = *reinterpret_cast<const float4 *>(&As[ra * DK + (((2 * h + s4) ^ ((ra >> 2) & 3)) << 2)]);
                b[i] = *reinterpret_cast<const float4 *>(&Bs[rb * DK + (((2 * h + s4) ^ ((rb >> 2) & 3)) << 2)]);
            }
#pragma unroll
            for (int e = 0; e < 4; ++e)
#pragma unroll
                for (int i = 0; i < 2; ++i)
#pragma unroll
                    for (int j = 0; j < 2; ++j) {
                        const float av = e == 0 ? a[i].x : e == 1 ? a[i].y : e == 2 ? a[i].z : a[i].w;
                        const float bv = e == 0 ? b[j].x : e == 1 ? b[j].y : e == 2 ? b[j].z : b[j].w;
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(bv, av, acc[i][j], 0, 0, 0);
                    }
        }
    }
    __syncthreads();   // operands are dead: the buffers may be reused
}

constexpr int SLD = 64 + 4;   // row stride (floats) of a wavefront's 32x64 output staging area in LDS

template <bool DMA>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(4, 4))) void coarse_gemm_kernel(
    const float *__restrict__ Q, const float *__restrict__ qn, int64_t nq,
    const float *__restrict__ C, const float *__restrict__ cn, int64_t K, int D,
    float *__restrict__ Dt, float *__restrict__ bm, int nb, int tiles_q)
{
    // operands (register-staged: two padded 128x32 tiles; DMA: two buffers of 256x16), reused as output staging
    __shared__ __attribute__((aligned(16))) float ops[DMA ? 4 * 32 * SLD : 2 * GT * GLD];
    static_assert(2 * DBUF <= 4 * 32 * SLD, "the DMA buffers must fit the staging area");
    __shared__ __attribute__((aligned(16))) float cns[GT];
    static_assert(4 * 32 * SLD <= 2 * GT * GLD, "the four staging areas must fit the operand buffers");
    float *As = ops, *Bs = ops + GT * GLD;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    int64_t q0, c0;
    if (!tile_of_block(blockIdx.x, tiles_q, q0, c0)) return;
    const int wq = (wave >> 1) * 64, wc = (wave & 1) * 64;
    const int l32 = lane & 31, h = lane >> 5;
    if (threadIdx.x < GT) cns[threadIdx.x] = c0 + threadIdx.x < K ? cn[c0 + threadIdx.x] : 0.f;
    floatx16 acc[2][2];
    // both end with a barrier: cns is visible, operands are dead
    if (DMA) gemm_tile_dma(Q, nq, q0, C, K, c0, D, ops, acc);
    else gemm_tile(Q, nq, q0, C, K, c0, D, As, Bs, acc);
    const bool vec = (K & 3) == 0;
    const int64_t blk = (c0 + wc) / BMW;
    float *stage = ops + wave * (32 * SLD);
    const int sr = lane >> 4, sc = (lane & 15) * 4;   // store phase: 16 lanes cover one query row of 64 centroids
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int64_t q = q0 + wq + i * 32 + l32;
        const float qr = q < nq ? qn[q] : 0.f;
        float m = INFINITY;
        // distances of 32 queries x 64 centroids into the staging area, [query][centroid]
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const int cl = j * 32 + 8 * g + 4 * h;          // centroid of element 4g inside the quadrant
                const int64_t c = c0 + wc + cl;
                const float4 cv = *reinterpret_cast<const float4 *>(&cns[wc + cl]);
                float4 d;
                d.x = fmaxf(fmaf(-2.f, acc[i][j][4 * g + 0], qr + cv.x), 0.f);
                d.y = fmaxf(fmaf(-2.f, acc[i][j][4 * g + 1], qr + cv.y), 0.f);
                d.z = fmaxf(fmaf(-2.f, acc[i][j][4 * g + 2], qr + cv.z), 0.f);
                d.w = fmaxf(fmaf(-2.f, acc[i][j][4 * g + 3], qr + cv.w), 0.f);
                m = fminf(m, c + 0 < K ? d.x : INFINITY);
                m = fminf(m, c + 1 < K ? d.y : INFINITY);
                m = fminf(m, c + 2 < K ? d.z : INFINITY);
                m = fminf(m, c + 3 < K ? d.w : INFINITY);
                *reinterpret_cast<float4 *>(&stage[l32 * SLD + cl]) = d;
            }
        m = fminf(m, __shfl_xor(m, 32, WAVE));   // the other half holds the other 32 centroids
        if (h == 0 && q < nq && blk < nb) bm[q * nb + blk] = m;
        wave_sync();
        // out again with 16 lanes per query row: every store instruction writes four rows of 256 contiguous bytes
#pragma unroll
        for (int it = 0; it < 8; ++it) {
            const int r = it * 4 + sr;
            const int64_t qq = q0 + wq + i * 32 + r, c = c0 + wc + sc;
            const float4 d = *reinterpret_cast<const float4 *>(&stage[r * SLD + sc]);
            if (qq < nq) {
                float *rowp = Dt + qq * K;
                if (vec && c + 3 < K) {
                    *reinterpret_cast<float4 *>(rowp + c) = d;
                } else {
                    const float dv[4] = {d.x, d.y, d.z, d.w};
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        if (c + e < K) rowp[c + e] = dv[e];
                }
            }
        }
        wave_sync();
    }
}

// The same for small batches (latency mode): a workgroup takes 32 queries x 256 centroids, all
// four wavefronts share the 32 queries and each owns 64 of the centroids (two accumulators),
// so a batch of up to 32 queries costs a quarter of the MFMA work of the 128-query tile and
// the kernel is bounded by streaming the centroid matrix once per 32 queries.
constexpr int SKQ = 32, SKC = 256;

__global__ __launch_bounds__(256) void coarse_gemm_skinny_kernel(
    const float *__restrict__ Q, const float *__restrict__ qn, int64_t nq,
    const float *__restrict__ C, const float *__restrict__ cn, int64_t K, int D,
    float *__restrict__ Dt, float *__restrict__ bm, int nb, int tiles_q)
{
    __shared__ __attribute__((aligned(16))) float ops[(SKQ + SKC) * GLD];   // operands; reused as output staging
    __shared__ __attribute__((aligned(16))) float cns[SKC];
    static_assert(4 * 32 * SLD <= (SKQ + SKC) * GLD, "the four staging areas must fit the operand buffers");
    float *As = ops, *Bs = ops + SKQ * GLD;
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int64_t q0 = (int64_t)(blockIdx.x % tiles_q) * SKQ, c0 = (int64_t)(blockIdx.x / tiles_q) * SKC;
    const int wc = wave * 64;
    const int l32 = lane & 31, h = lane >> 5;
    cns[tid] = c0 + tid < K ? cn[c0 + tid] : 0.f;
    floatx16 acc[2];
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[j][v] = 0.f;
    float4 pa, pb[8];
    auto fetch = [&](int k0) {
        const int c4 = (tid & 7) * 4;
        pa = make_float4(0.f, 0.f, 0.f, 0.f);
        if (k0 + c4 < D && q0 + (tid >> 3) < nq)
            pa = *reinterpret_cast<const float4 *>(Q + (q0 + (tid >> 3)) * D + k0 + c4);
#pragma unroll
        for (int it = 0; it < 8; ++it) {
            const int row = (tid >> 3) + it * 32;
            pb[it] = make_float4(0.f, 0.f, 0.f, 0.f);
            if (k0 + c4 < D && c0 + row < K)
                pb[it] = *reinterpret_cast<const float4 *>(C + (c0 + row) * D + k0 + c4);
        }
    };
    fetch(0);
    for (int k0 = 0; k0 < D; k0 += GKC) {
        const int c4 = (tid & 7) * 4;
        *reinterpret_cast<float4 *>(&As[(tid >> 3) * GLD + c4]) = pa;
#pragma unroll
        for (int it = 0; it < 8; ++it)
            *reinterpret_cast<float4 *>(&Bs[((tid >> 3) + it * 32) * GLD + c4]) = pb[it];
        __syncthreads();
        if (k0 + GKC < D) fetch(k0 + GKC);
#pragma unroll
        for (int s4 = 0; s4 < 4; ++s4) {
            const int kc = (s4 >> 1) * 16 + h * 8 + (s4 & 1) * 4;   // same k order as the other variants
            const float4 a = *reinterpret_cast<const float4 *>(&As[l32 * GLD + kc]);
            float4 b[2];
#pragma unroll
            for (int j = 0; j < 2; ++j)
                b[j] = *reinterpret_cast<const float4 *>(&Bs[(wc + j * 32 + l32) * GLD + kc]);
#pragma unroll
            for (int e = 0; e < 4; ++e)
#pragma unroll
                for (int j = 0; j < 2; ++j) {
                    const float av = e == 0 ? a.x : e == 1 ? a.y : e == 2 ? a.z : a.w;
                    const float bv = e == 0 ? b[j].x : e == 1 ? b[j].y : e == 2 ? b[j].z : b[j].w;
                    acc[j] = __builtin_amdgcn_mfma_f32_32x32x2f32(bv, av, acc[j], 0, 0, 0);
                }
        }
        __syncthreads();
    }
    const bool vec = (K & 3) == 0;
    const int64_t blk = (c0 + wc) / BMW;
    float *stage = ops + wave * (32 * SLD);
    const int sr = lane >> 4, sc = (lane & 15) * 4;
    const int64_t q = q0 + l32;
    const float qr = q < nq ? qn[q] : 0.f;
    float m = INFINITY;
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            const int cl = j * 32 + 8 * g + 4 * h;
            const int64_t c = c0 + wc + cl;
            const float4 cv = *reinterpret_cast<const float4 *>(&cns[wc + cl]);
            float4 d;
            d.x = fmaxf(fmaf(-2.f, acc[j][4 * g + 0], qr + cv.x), 0.f);
            d.y = fmaxf(fmaf(-2.f, acc[j][4 * g + 1], qr + cv.y), 0.f);
            d.z = fmaxf(fmaf(-2.f, acc[j][4 * g + 2], qr + cv.z), 0.f);
            d.w = fmaxf(fmaf(-2.f, acc[j][4 * g + 3], qr + cv.w), 0.f);
            m = fminf(m, c + 0 < K ? d.x : INFINITY);
            m = fminf(m, c + 1 < K ? d.y : INFINITY);
            m = fminf(m, c + 2 < K ? d.z : INFINITY);
            m = fminf(m, c + 3 < K ? d.w : INFINITY);
            *reinterpret_cast<float4 *>(&stage[l32 * SLD + cl]) = d;
        }
    m = fminf(m, __shfl_xor(m, 32, WAVE));
    if (h == 0 && q < nq && blk < nb) bm[q * nb + blk] = m;
    wave_sync();
#pragma unroll
    for (int it = 0; it < 8; ++it) {
        const int r = it * 4 + sr;
        const int64_t qq = q0 + r, c = c0 + wc + sc;
        const float4 d = *reinterpret_cast<const float4 *>(&stage[r * SLD + sc]);
        if (qq < nq) {
            float *rowp = Dt + qq * K;
            if (vec && c + 3 < K) {
                *reinterpret_cast<float4 *>(rowp + c) = d;
            } else {
                const float dv[4] = {d.x, d.y, d.z, d.w};
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    if (c + e < K) rowp[c + e] = dv[e];
            }
        }
    }
}

// Nearest centroid only (P = 1): the same tile product, reduced on the fly to
// the per-query minimum of (distance, centroid id), merged across centroid
// tiles with a 64-bit atomic minimum; no distance tile is written.  best[]
// must be pre-filled with all ones.
__global__ __launch_bounds__(256) void coarse_argmin_kernel(
    const float *__restrict__ Q, const float *__restrict__ qn, int64_t nq,
    const float *__restrict__ C, const float *__restrict__ cn, int64_t K, int D,
    unsigned long long *__restrict__ best, int tiles_q)
{
    __shared__ __attribute__((aligned(16))) float As[GT * GLD];
    __shared__ __attribute__((aligned(16))) float Bs[GT * GLD];
    __shared__ __attribute__((aligned(16))) float cns[GT];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    int64_t q0, c0;
    if (!tile_of_block(blockIdx.x, tiles_q, q0, c0)) return;
    const int wq = (wave >> 1) * 64, wc = (wave & 1) * 64;
    const int l32 = lane & 31, h = lane >> 5;
    if (threadIdx.x < GT) cns[threadIdx.x] = c0 + threadIdx.x < K ? cn[c0 + threadIdx.x] : 0.f;
    floatx16 acc[2][2];
    gemm_tile(Q, nq, q0, C, K, c0, D, As, Bs, acc);
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int64_t q = q0 + wq + i * 32 + l32;
        const float qr = q < nq ? qn[q] : 0.f;
        unsigned long long key = ~0ull;
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int cl = wc + j * 32 + 8 * (v >> 2) + 4 * h + (v & 3);
                const int64_t c = c0 + cl;
                if (c < K) {
                    float d = fmaxf(fmaf(-2.f, acc[i][j][v], qr + cns[cl]), 0.f);
                    unsigned long long kc = ((unsigned long long)float_key(d) << 32) | (uint32_t)c;
                    key = kc < key ? kc : key;
                }
            }
        unsigned long long other = __shfl_xor(key, 32, WAVE);
        key = other < key ? other : key;
        if (h == 0 && q < nq) atomicMin(&best[q], key);
    }
}

__global__ __launch_bounds__(256) void argmin_unpack_kernel(const unsigned long long *__restrict__ best,
                                                            int64_t n, int32_t *__restrict__ out_id,
                                                            float *__restrict__ out_d)
{
    int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= n) return;
    unsigned long long k = best[i];
    out_id[i] = (int32_t)(uint32_t)k;
    if (out_d) out_d[i] = key_float((uint32_t)(k >> 32));
}

// The P closest centroids of each query row of Dt by (distance, id), written
// in ascending centroid id.  One workgroup per query, in three steps:
//   1. t = the min(P, nb)-th smallest block minimum.  The P smallest block
//      minima are P distinct distances <= t, so every one of the P closest
//      centroids has distance <= t and lies in a block whose minimum is <= t.
//   2. list, in ascending order, every block with minimum < t (fewer than P)
//      and the first P blocks with minimum == t (a later such block is
//      preceded by at least P distances equal to t, so it cannot contribute).
//   3. exact radix select of the P smallest (distance, id) among the
//      elements of the listed blocks (at most 2P*64), read from Dt.
// blist is dynamic LDS of 2*P ints.
template <int BLOCK>
__global__ __launch_bounds__(BLOCK) void probe_select_kernel(const float *__restrict__ Dt,
                                                             const float *__restrict__ bm, int64_t K,
                                                             int nb, int P,
                                                             int32_t *__restrict__ probe_id,
                                                             float *__restrict__ probe_d)
{
    __shared__ SelectShared sh;
    __shared__ uint32_t nflag_s;
    extern __shared__ int blist[];
    const int64_t q = blockIdx.x;
    const float *row = Dt + q * K;
    const float *bmr = bm + q * nb;
    auto keyb = [bmr](int64_t b) { return float_key(bmr[b]); };
    const uint32_t nselb = P < nb ? (uint32_t)P : (uint32_t)nb;
    uint32_t t, needb;
    block_radix_select<BLOCK>(keyb, nb, nselb, sh, t, needb);
    uint32_t nflag = block_emit_selected<BLOCK>(keyb, nb, 0xFFFFFFFFu, t, (uint32_t)P, sh,
                                                [&](uint32_t pos, int64_t b, uint32_t) { blist[pos] = (int)b; });
    if (threadIdx.x == 0) nflag_s = nflag;
    __syncthreads();
    nflag = nflag_s;
    auto keyv = [row, K](int64_t v, const int *bl) {
        int64_t c = (int64_t)bl[v >> 6] * BMW + (v & 63);
        return c < K ? float_key(row[c]) : 0xFFFFFFFFu;
    };
    auto key = [&](int64_t v) { return keyv(v, blist); };
    uint32_t pivot, need;
    block_radix_select<BLOCK>(key, (int64_t)nflag * BMW, (uint32_t)P, sh, pivot, need);
    block_emit_selected<BLOCK>(key, (int64_t)nflag * BMW, (uint32_t)P, pivot, need, sh,
                               [&](uint32_t pos, int64_t v, uint32_t k) {
                                   probe_id[q * P + pos] = blist[v >> 6] * BMW + (int)(v & 63);
                                   probe_d[q * P + pos] = key_float(k);
                               });
}

}  // namespace ivf
