// Stage 1: squared distances from a tile of queries to all K centroids as an
// MFMA GEMM (||q||^2 - 2<q,c> + ||c||^2), and the exact per-query selection of
// the nprobe closest regions (exhaustive assignment, Section 3.1).
//
// The inner products run on the fp16 matrix cores at fp32 accuracy: every
// operand row is scaled by a power of two so that its largest magnitude lies in
// [2^14, 2^15) and split into hi = fp16(x) and lo = fp16(x - hi), which
// together carry 22 significant bits; <q,c> is accumulated in fp32 from the
// three products lo*hi + hi*lo + hi*hi per 16 dimensions (each fp16 product is
// exact in fp32; the dropped lo*lo term is below 2^-24 of |q_i c_i|), and the
// scales, being powers of two, are undone exactly in the epilogue.  The
// rounding error of a distance is that of an fp32 dot product with 18 instead
// of 96 accumulation steps.
#pragma once
#include "select.hpp"

namespace ivf {

typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef _Float16 halfx8 __attribute__((ext_vector_type(8)));
typedef uint32_t gu32x4 __attribute__((ext_vector_type(4)));

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

// Largest magnitude of count floats, as the bit pattern of a non-negative float
// (those order like unsigned integers); out must start at 0.
__global__ __launch_bounds__(256) void absmax_kernel(const float *__restrict__ X, int64_t count,
                                                     uint32_t *__restrict__ out)
{
    float m = 0.f;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < count; i += (int64_t)gridDim.x * 256)
        m = fmaxf(m, fabsf(X[i]));
#pragma unroll
    for (int o = WAVE / 2; o > 0; o >>= 1) m = fmaxf(m, __shfl_xor(m, o, WAVE));
    if ((threadIdx.x & 63) == 0) atomicMax(out, __float_as_uint(m));
}

constexpr int DK = 16;                       // dimensions per operand stage
// packed width of a row: whole stages, and an even number of them (the GEMM loops are unrolled by two)
__host__ __device__ inline int packed_dim(int D) { return (D + 2 * DK - 1) / (2 * DK) * (2 * DK); }
// Rows a packed matrix of n rows must be allocated for: the GEMM tiles copy whole tiles of up
// to 256 rows without clamping (rows past n are read, their products are never stored).
__host__ __device__ inline int64_t packed_rows(int64_t n) { return (n + 255) / 256 * 256; }

// Operand packing for the GEMM: row r of X ([n][D] fp32) becomes packed_dim(D)/16
// (an even number of) stages of 64 bytes, stage t = [hi k0..7 | lo k0..7 | hi k8..15 | lo k8..15] of
// dimensions 16t + k (fp16, zero beyond D), scaled by s = 2^(14 - floor(log2 m)):
// m is the row's largest magnitude, or the whole matrix's when gmax (the result
// of absmax_kernel) is given.  Also writes ||row||^2 and 1/s (per row, or
// inv_scale[0] for a matrix-wide scale).  One wavefront per row.
__global__ __launch_bounds__(256) void split_rows_kernel(const float *__restrict__ X, int64_t n, int D,
                                                         const uint32_t *__restrict__ gmax,
                                                         _Float16 *__restrict__ P, float *__restrict__ norm,
                                                         float *__restrict__ inv_scale)
{
    const int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    const int lane = threadIdx.x & 63;
    if (row >= n) return;
    const int Dp = packed_dim(D);
    float s2 = 0.f, m = 0.f;
    for (int i = lane; i < D; i += WAVE) {
        const float v = X[row * D + i];
        s2 = fmaf(v, v, s2);
        m = fmaxf(m, fabsf(v));
    }
    s2 = wave_sum(s2);
    if (gmax) {
        m = __uint_as_float(*gmax);
    } else {
#pragma unroll
        for (int o = WAVE / 2; o > 0; o >>= 1) m = fmaxf(m, __shfl_xor(m, o, WAVE));
    }
    int e = (m > 0.f && m < INFINITY) ? ilogbf(m) : 14;
    e = e < -100 ? -100 : e > 100 ? 100 : e;
    const float s = ldexpf(1.f, 14 - e);
    _Float16 *out = P + row * (int64_t)Dp * 2;
    for (int i = lane; i < Dp; i += WAVE) {
        const float v = i < D ? X[row * D + i] * s : 0.f;
        const _Float16 hi = (_Float16)v;
        const _Float16 lo = (_Float16)(v - (float)hi);
        const int at = (i >> 4) * 32 + ((i >> 3) & 1) * 16 + (i & 7);
        out[at] = hi;
        out[at + 8] = lo;
    }
    if (lane == 0) {
        norm[row] = s2;
        if (!gmax) inv_scale[row] = ldexpf(1.f, e - 14);
        else if (row == 0) inv_scale[0] = ldexpf(1.f, e - 14);
    }
}

constexpr int GT = 128;        // tile: GT queries x GT centroids per workgroup
constexpr int DBUF = 2 * GT * DK;            // floats per operand buffer (A rows then B rows)
constexpr int ROWF = DK;                     // floats (4-byte units) per packed row stage: 64 bytes

// acc += <A row, B row> over one staged 16 dimensions for this lane's fragments:
// a[0]/b[0] hold hi, a[1]/b[1] lo of the lane half's 8 dimensions.  The small
// cross terms go first.  The centroids are the MFMA's row operand.
__device__ __forceinline__ floatx16 mfma3(const gu32x4 (&bfrag)[2], const gu32x4 (&afrag)[2], floatx16 acc, int which)
{
    const halfx8 bh = __builtin_bit_cast(halfx8, bfrag[0]), bl = __builtin_bit_cast(halfx8, bfrag[1]);
    const halfx8 ah = __builtin_bit_cast(halfx8, afrag[0]), al = __builtin_bit_cast(halfx8, afrag[1]);
    if (which == 0) return __builtin_amdgcn_mfma_f32_32x32x16_f16(bl, ah, acc, 0, 0, 0);
    if (which == 1) return __builtin_amdgcn_mfma_f32_32x32x16_f16(bh, al, acc, 0, 0, 0);
    return __builtin_amdgcn_mfma_f32_32x32x16_f16(bh, ah, acc, 0, 0, 0);
}

// One 128x128 tile of <Q[q], C[j]> per workgroup of 4 wavefronts; each
// wavefront owns a 64x64 quadrant as 2x2 v_mfma_f32_32x32x16_f16 accumulators.
// Operands are the packed rows above, copied global -> LDS by
// global_load_lds_dwordx4 (no registers, no ds_write) in stages of 16
// dimensions, two LDS buffers so that the copy of stage s+1 runs under the MFMA
// block of stage s with one barrier per stage.  A direct-to-LDS load puts lane
// i's 16 bytes at base + 16 i, so the layout is unpadded rows of four 16-byte
// chunks; bank conflicts of the operand reads are avoided by storing chunk f of
// row r in slot f ^ ((r >> 2) & 3) (each lane simply fetches the chunk that
// belongs to its slot).  Lane half h feeds dimensions [8h, 8h+8) of the stage:
// chunks 2h (hi) and 2h+1 (lo).  All variants of the kernel use this k order,
// so a query's distances do not depend on the batch it arrives in.
// In acc[i][j], lane l holds query (column) wq + 32i + l%32 and element v is
// centroid (row) wc + 32j + 8*(v/4) + 4*(l/32) + v%4, i.e. four groups of four
// consecutive centroids, which the epilogues store as 128-bit words and reduce
// without leaving the lane.  buf0 and buf1 each hold (128 + 128) rows x 64 bytes.
//
// HI = true: the operands are the hi-only tables of pack_hi_kernel (a row stage of 64 bytes holds 32
// dimensions: for lane half h the chunks 2h and 2h+1 are its 8 dimensions of the stage's first and
// second 16), Dp is that table's row length in 4-byte units, and a stage is two products hi*hi: a
// third of the MFMA work and half the bytes for an approximation of <q,c> whose error the caller bounds.
template <bool HI = false>
__device__ __forceinline__ void gemm_tile(const _Float16 *__restrict__ Qp, int64_t nq, int64_t q0,
                                          const _Float16 *__restrict__ Cp, int64_t K, int64_t c0, int Dp,
                                          float *buf0, float *buf1, floatx16 (&acc)[2][2])
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

    // This wave's four copies per stage: 16-row blocks 4 wave .. 4 wave + 3 of the buffer, i.e. 64
    // consecutive rows of one operand (waves 0-1 the query rows, 2-3 the centroid rows).  Both
    // packed matrices are allocated up to a multiple of the tile height, so no row is clamped
    // (products of rows past the end are never stored), and the copies are one instruction in a
    // rolled loop: the compiler tracks only a handful of distinct LDS copies exactly.
    const int r0 = (wave & 1) * 64 + (lane >> 2);                      // first row inside the operand tile
    const int f = (lane & 3) ^ ((r0 >> 2) & 3);                        // chunk this slot holds (same for all four rows)
    const float *src0 = wave < 2 ? reinterpret_cast<const float *>(Qp) + (q0 + r0) * Dp + f * 4
                                 : reinterpret_cast<const float *>(Cp) + (c0 + r0) * Dp + f * 4;
    auto issue = [&](int k0, float *dst) {
#pragma nounroll
        for (int n = 0; n < 4; ++n)
            __builtin_amdgcn_global_load_lds((gptr_t)(src0 + (int64_t)n * 16 * Dp + k0),
                                             (lptr_t)(dst + (wave * 4 + n) * 256), 16, 0, 0);
    };
    auto compute = [&](const float *As) {
        const float *Bs = As + GT * ROWF;
        gu32x4 a[2][2], b[2][2];
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int ra = wq + i * 32 + l32, rb = wc + i * 32 + l32;
#pragma unroll
            for (int p = 0; p < 2; ++p) {
                a[i][p] = *reinterpret_cast<const gu32x4 *>(&As[ra * ROWF + (((2 * h + p) ^ ((ra >> 2) & 3)) << 2)]);
                b[i][p] = *reinterpret_cast<const gu32x4 *>(&Bs[rb * ROWF + (((2 * h + p) ^ ((rb >> 2) & 3)) << 2)]);
            }
        }
        // the four accumulators are independent: cycle through them so that no MFMA
        // waits for the one issued just before it
        if (HI) {
#pragma unroll
            for (int p = 0; p < 2; ++p)
#pragma unroll
                for (int i = 0; i < 2; ++i)
#pragma unroll
                    for (int j = 0; j < 2; ++j)
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(halfx8, b[j][p]),
                                                                           __builtin_bit_cast(halfx8, a[i][p]), acc[i][j], 0, 0, 0);
        } else {
#pragma unroll
            for (int e = 0; e < 3; ++e)
#pragma unroll
                for (int i = 0; i < 2; ++i)
#pragma unroll
                    for (int j = 0; j < 2; ++j) acc[i][j] = mfma3(b[j], a[i], acc[i][j], e);
        }
    };
    // The two buffers are separate LDS objects and every step names them statically (the loop
    // is unrolled by two): the compiler can then tell that the operand reads of one buffer do
    // not depend on the copy in flight into the other, and leaves that copy running under the
    // MFMA block.
    const int stages = Dp / DK;               // (even for the hi/lo tables, any number for the hi-only ones)
    issue(0, buf0);
    for (int s = 0; s < stages; s += 2) {
        __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0): this wave's copies of stage s have landed
        __syncthreads();                      // ... and everyone's; all waves are done with the other buffer
        if (s + 1 < stages) issue((s + 1) * DK, buf1);
        compute(buf0);
        if (s + 1 < stages) {
            __builtin_amdgcn_s_waitcnt(0x0F70);
            __syncthreads();
            if (s + 2 < stages) issue((s + 2) * DK, buf0);
            compute(buf1);
        }
    }
    __syncthreads();   // operands are dead: the buffers may be reused
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

constexpr int SLD = 64 + 4;   // row stride (floats) of a wavefront's 32x64 output staging area in LDS

// Epilogue of one 32-query x 64-centroid block held by a wavefront as two accumulators
// (acc[j]: centroids 32j .. 32j+31 of the block): distances max(0, qr + cn + m2 * acc), the
// block minimum per query into bm (BM_LDS: into the LDS word bm_lds[query of the block * bm_lds_stride]),
// and the distances out through the wavefront's LDS staging
// area, [query][centroid], so that 16 lanes cover one query row and every store instruction
// writes four rows of 256 contiguous bytes, as streaming (non-temporal) stores: the matrix is
// far larger than the caches and is read back by other kernels only after this one has ended,
// and on the MI355X the sweep kernel runs 10 % faster with them than with ordinary stores.
// qb / cb: first query / centroid of the block;
// cnw: the 64 centroid norms of the block (LDS).  EDGE = false skips all bounds checks (the
// block lies inside Dt and K is a multiple of 4).
template <bool EDGE, int SROWS = 32, bool BM_LDS = false>
__device__ __forceinline__ void emit_block(const floatx16 (&acc)[2], float qr, float m2, const float *cnw,
                                           float *stage, int64_t qb, int64_t nq, int64_t cb, int64_t K,
                                           float *__restrict__ Dt, int64_t ldt, float *__restrict__ bm, int nb,
                                           float *bm_lds = nullptr, int bm_lds_stride = 0)
{
    static_assert(SROWS == 32 || SROWS == 16, "the staging area holds 32 or 16 query rows");
    const int lane = threadIdx.x & 63;
    const int l32 = lane & 31, h = lane >> 5;
    const int sr = lane >> 4, sc = (lane & 15) * 4;
    float4 d[2][4];
    float m = INFINITY;
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            const int cl = j * 32 + 8 * g + 4 * h;          // centroid of element 4g inside the block
            const float4 cv = *reinterpret_cast<const float4 *>(&cnw[cl]);
            float4 &e = d[j][g];
            e.x = fmaxf(fmaf(m2, acc[j][4 * g + 0], qr + cv.x), 0.f);
            e.y = fmaxf(fmaf(m2, acc[j][4 * g + 1], qr + cv.y), 0.f);
            e.z = fmaxf(fmaf(m2, acc[j][4 * g + 2], qr + cv.z), 0.f);
            e.w = fmaxf(fmaf(m2, acc[j][4 * g + 3], qr + cv.w), 0.f);
            if (EDGE) {
                const int64_t c = cb + cl;
                m = fminf(m, c + 0 < K ? e.x : INFINITY);
                m = fminf(m, c + 1 < K ? e.y : INFINITY);
                m = fminf(m, c + 2 < K ? e.z : INFINITY);
                m = fminf(m, c + 3 < K ? e.w : INFINITY);
            } else {
                m = fminf(fminf(m, e.x), fminf(e.y, fminf(e.z, e.w)));
            }
        }
    m = fminf(m, __shfl_xor(m, 32, WAVE));   // the other half holds the other 32 centroids
    const int64_t q = qb + l32, blk = cb / BMW;
    if (BM_LDS) {   // the caller collects the minima of several blocks and writes them out as whole sectors
        // (an explicit instruction: before an ordinary LDS write the compiler may wait for every
        // outstanding vector-memory operation when direct-to-LDS copies are in flight)
        const uint32_t at = (uint32_t)reinterpret_cast<uintptr_t>(bm_lds + l32 * bm_lds_stride);   // LDS byte address
        if (h == 0) asm volatile("ds_write_b32 %0, %1" ::"v"(at), "v"(m) : "memory");
    } else if (h == 0 && (!EDGE || (q < nq && blk < nb))) {
        bm[q * nb + blk] = m;
    }
    // through the staging area, SROWS query rows at a time (the lanes of the other rows sit a pass out).
    // The interior path issues exactly (32 / SROWS) * (SROWS / 4) store instructions: the sweep kernel's
    // hand-counted waits depend on that number.
#pragma unroll
    for (int pass = 0; pass < 32 / SROWS; ++pass) {
        if (SROWS == 32 || (l32 / SROWS) == pass) {
#pragma unroll
            for (int j = 0; j < 2; ++j)
#pragma unroll
                for (int g = 0; g < 4; ++g)
                    *reinterpret_cast<float4 *>(&stage[(l32 % SROWS) * SLD + j * 32 + 8 * g + 4 * h]) = d[j][g];
        }
        wave_sync();
        const int64_t qp = qb + pass * SROWS;
        if (EDGE) {
            const bool vec = (K & 3) == 0;
#pragma unroll
            for (int it = 0; it < SROWS / 4; ++it) {
                const int r = it * 4 + sr;
                const int64_t qq = qp + r, c = cb + sc;
                const float4 v = *reinterpret_cast<const float4 *>(&stage[r * SLD + sc]);
                if (qq < nq) {
                    float *rowp = Dt + qq * ldt;
                    if (vec && c + 3 < K) {
                        *reinterpret_cast<float4 *>(rowp + c) = v;
                    } else {
                        const float dv[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
                        for (int e = 0; e < 4; ++e)
                            if (c + e < K) rowp[c + e] = dv[e];
                    }
                }
            }
        } else {
            float *p = Dt + (qp + sr) * ldt + cb + sc;
#pragma unroll
            for (int it = 0; it < SROWS / 4; ++it) {
                __builtin_nontemporal_store(*reinterpret_cast<const floatx4 *>(&stage[(it * 4 + sr) * SLD + sc]),
                                            reinterpret_cast<floatx4 *>(p));
                p += 4 * ldt;
            }
        }
        wave_sync();
    }
}

// Row stride of the distance matrix Dt in floats.  Unpadded: padding the rows (by 128 bytes up
// to 16 KB) made the tile stores slower on the MI355X, not faster.
__host__ __device__ inline int64_t dt_stride(int64_t K) { return K; }

// Dt[q][j] = max(0, qn[q] + cn[j] - 2 <Q[q], C[j]>), and bm[q][b] = the minimum
// of Dt[q][64b .. 64b+63] (each wavefront's 64-centroid quadrant gives one block
// minimum per query).  qsi[q] and csi[0] are the inverse operand scales.  The
// grid has 8 * ceil(tiles_q / 8) * tiles_c workgroups.
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(4, 4))) void coarse_gemm_kernel(
    const _Float16 *__restrict__ Qp, const float *__restrict__ qn, const float *__restrict__ qsi, int64_t nq,
    const _Float16 *__restrict__ Cp, const float *__restrict__ cn, const float *__restrict__ csi, int64_t K,
    int Dp, float *__restrict__ Dt, int64_t ldt, float *__restrict__ bm, int nb, int tiles_q)
{
    // two operand buffers of 256 rows x 64 bytes, each reused as the output staging of two wavefronts
    __shared__ __attribute__((aligned(16))) float ops0[2 * 32 * SLD];
    __shared__ __attribute__((aligned(16))) float ops1[2 * 32 * SLD];
    static_assert(DBUF <= 2 * 32 * SLD, "an operand buffer must fit the staging area of two wavefronts");
    __shared__ __attribute__((aligned(16))) float cns[GT];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    int64_t q0, c0;
    if (!tile_of_block(blockIdx.x, tiles_q, q0, c0)) return;
    const int wq = (wave >> 1) * 64, wc = (wave & 1) * 64;
    const int l32 = lane & 31, h = lane >> 5;
    if (threadIdx.x < GT) cns[threadIdx.x] = c0 + threadIdx.x < K ? cn[c0 + threadIdx.x] : 0.f;
    floatx16 acc[2][2];
    gemm_tile(Qp, nq, q0, Cp, K, c0, Dp, ops0, ops1, acc);   // ends with a barrier: cns is visible, operands are dead
    const float m2c = -2.f * csi[0];
    float *stage = (wave < 2 ? ops0 : ops1) + (wave & 1) * (32 * SLD);
    const bool interior = q0 + GT <= nq && c0 + GT <= K && (K & 3) == 0;   // uniform over the workgroup
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int64_t qb = q0 + wq + i * 32, q = qb + l32;
        const float qr = q < nq ? qn[q] : 0.f;
        const float m2 = q < nq ? m2c * qsi[q] : 0.f;
        if (interior) emit_block<false>(acc[i], qr, m2, cns + wc, stage, qb, nq, c0 + wc, K, Dt, ldt, bm, nb);
        else emit_block<true>(acc[i], qr, m2, cns + wc, stage, qb, nq, c0 + wc, K, Dt, ldt, bm, nb);
    }
}

// s_waitcnt immediate that waits until at most n vector-memory operations of the wavefront are
// outstanding (they complete in issue order) and leaves the other counters alone.
constexpr int vmcnt_imm(int n) { return (n & 15) | ((n >> 4) << 14) | (7 << 4) | (15 << 8); }

// Large batches, STAGES = packed_dim / 16 known at compile time: a workgroup keeps ONE query
// tile and sweeps `tiles_per_wg` consecutive centroid tiles.  Its query operand never passes
// through LDS: every lane holds the fragments of its query rows for all stages in registers
// (16 STAGES of them), so per centroid tile only the 128 centroid rows are copied
// (global -> LDS, 8 KB a stage) into a ring of RING buffers, PD = RING - 1 stages ahead (a copy
// takes a few microseconds to land, several steps' worth of MFMA work), and
// the ring keeps running across tiles: the copies of the next tile's first stages are in
// flight during the epilogue of the current one.  The distance stores of a workgroup walk
// along its 128 rows of Dt, tile after tile.  STAGES is a multiple of RING, so stage s of
// every tile uses buffer s % RING and each step names its buffer statically (separate LDS
// objects, see gemm_tile).  Same k order and products as gemm_tile: identical results.
//
// Waiting for a copy with operations issued after it still in flight relies on in-order
// completion; the counts below are the vector-memory operations a wavefront issues between a
// copy and the step that consumes it, or a lower bound of them (2 copies a step, at least 16
// stores an epilogue).  With six stages the ring holds a whole tile and every copy is issued
// ahead of the stores of the tile before the one it belongs to: a wavefront never has to wait
// for its stores to drain before it can go on, it runs up to one tile ahead of them.  Only whole
// tiles are handled (K a multiple of 128; the rows of a partial last query tile are computed
// too, into the padding of the per-query buffers).  The workgroup barrier of a step orders LDS
// traffic only (operands arrive by copies that each wavefront has waited for, nothing else is
// shared), so it is issued without the global-memory fence of __syncthreads, which would drain
// the queue at every step.
//
// Block minima: a tile gives every query two of them (one per 64-centroid half), 4 bytes each in
// 128 different rows of bm.  Written directly, those scattered words took a third of the
// kernel's store-path cycles; they are collected in LDS for SWEEP_BMC consecutive tiles instead
// and written as 64-byte pieces (16 consecutive blocks of a row).
constexpr int SWEEP_BMC = 8;   // tiles per write-out of the block minima

template <int STAGES>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2, 2))) void coarse_gemm_sweep_kernel(
    const _Float16 *__restrict__ Qp, const float *__restrict__ qn, const float *__restrict__ qsi, int64_t nq,
    const _Float16 *__restrict__ Cp, const float *__restrict__ cn, const float *__restrict__ csi, int64_t K,
    float *__restrict__ Dt, int64_t ldt, float *__restrict__ bm, int nb, int tiles_q, int tiles_c, int tiles_per_wg)
{
    typedef const __attribute__((address_space(1))) void *gptr_t;
    typedef __attribute__((address_space(3))) void *lptr_t;
    constexpr int RING = STAGES <= 6 ? STAGES : 4;        // 6 stages: the ring holds a whole tile
    static_assert(STAGES % RING == 0 && STAGES >= RING && RING <= 6, "stage s of every tile must use buffer s % RING");
    constexpr int PD = RING - 1;
    constexpr int Dp = STAGES * DK;
    constexpr int SLOT = GT * ROWF;                        // floats per ring buffer: 128 rows x 64 bytes
    // Distance stores of one tile's interior epilogue per wavefront: two emit_block<false, SROWS = 16, true>
    // calls, each 32 / SROWS passes of SROWS / 4 store instructions for its two 32-centroid halves' 64
    // columns (one instruction covers 4 rows x 256 bytes).  The waits below count on exactly this number
    // of vector-memory operations between a copy and its consumer: emit_block's store count is part of
    // this kernel's contract.
    constexpr int EPI_SROWS = 16;
    constexpr int EPI_STORES = 2 * (32 / EPI_SROWS) * (EPI_SROWS / 4);
    static_assert(EPI_STORES == 16, "the vmcnt immediates of the sweep loop assume 16 epilogue stores per tile");
    __shared__ __attribute__((aligned(16))) float ring0[SLOT];
    __shared__ __attribute__((aligned(16))) float ring1[SLOT];
    __shared__ __attribute__((aligned(16))) float ring2[SLOT];
    __shared__ __attribute__((aligned(16))) float ring3[RING > 3 ? SLOT : 4];
    __shared__ __attribute__((aligned(16))) float ring4[RING > 4 ? SLOT : 4];
    __shared__ __attribute__((aligned(16))) float ring5[RING > 5 ? SLOT : 4];
    __shared__ __attribute__((aligned(16))) float stage_all[4 * 16 * SLD];   // 16 query rows per wavefront at a time
    __shared__ __attribute__((aligned(16))) float cns[2][GT];
    constexpr int BMC = SWEEP_BMC, BMLD = 2 * BMC + 4;     // row stride of the collected minima (floats)
    __shared__ __attribute__((aligned(16))) float bmbuf[GT * BMLD];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l32 = lane & 31, h = lane >> 5;
    const int wq = (wave >> 1) * 64, wc = (wave & 1) * 64;

    // workgroup -> (query tile, range of centroid tiles): XCD x = b % 8 owns query tiles x, x+8, ...;
    // step t of the workgroup is centroid tile tb + t
    const int tq_per = (tiles_q + N_XCD - 1) / N_XCD;
    const int xcd = (int)(blockIdx.x % N_XCD);
    const int64_t local = blockIdx.x / N_XCD;
    const int tq = (int)(local % tq_per) * N_XCD + xcd;
    if (tq >= tiles_q) return;
    const int tb = (int)(local / tq_per) * tiles_per_wg;    // a multiple of SWEEP_BMC (the host's tiles_per_wg is)
    const int t_begin = 0;
    int t_end = tb < tiles_c ? tiles_c - tb : 0;            // steps inside the matrix
    if (t_end > tiles_per_wg) t_end = tiles_per_wg;
    if (t_begin >= t_end) return;
    const int64_t q0 = (int64_t)tq * GT;

    // this wave's two copies per stage: rows 32 wave + 16 n + lane / 4 of the centroid tile
    const int rl = wave * 32 + (lane >> 2);
    const int fl = (lane & 3) ^ ((lane >> 4) & 3);         // ((row >> 2) & 3 is the same for both rows)
    const float *cbase = reinterpret_cast<const float *>(Cp) + (int64_t)rl * Dp + fl * 4;
    auto slot_of = [&](int s) -> float * {
        const int r = s % RING;
        return r == 0 ? ring0 : r == 1 ? ring1 : r == 2 ? ring2 : r == 3 ? ring3 : r == 4 ? ring4 : ring5;
    };
    // copy stage s (may be >= STAGES: a stage of the following tile) of tile t; past the range the
    // last tile is copied again (never read), so that the number of copies per step is fixed
    auto issue = [&](int t, int s) {
        if (s >= STAGES) { s -= STAGES; ++t; }
        if (t >= t_end) t = t_end - 1;
        const float *src = cbase + (int64_t)(tb + t) * GT * Dp + s * DK;
        float *dst = slot_of(s) + wave * 512;
#pragma nounroll
        for (int n = 0; n < 2; ++n)
            __builtin_amdgcn_global_load_lds((gptr_t)(src + (int64_t)n * 16 * Dp), (lptr_t)(dst + n * 256), 16, 0, 0);
    };

    // RING == STAGES: the ring holds one whole tile; the copy of a stage of the next tile is issued
    // one step after that stage was consumed, and the last one right after the tile's MFMA work,
    // ahead of the epilogue's stores, so that no copy ever queues behind a store it is needed before.
    constexpr bool WHOLE = RING == STAGES;
#pragma unroll
    for (int s = 0; s < (WHOLE ? STAGES : PD); ++s) issue(t_begin, s);

    // query fragments: for stage s and block i the 32 bytes [hi | lo] of row wq + 32 i + l32, half h
    gu32x4 afr[STAGES][2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const gu32x4 *row = reinterpret_cast<const gu32x4 *>(reinterpret_cast<const float *>(Qp) + (q0 + wq + i * 32 + l32) * Dp) + 2 * h;
#pragma unroll
        for (int s = 0; s < STAGES; ++s) {
            afr[s][i][0] = row[s * 4 + 0];
            afr[s][i][1] = row[s * 4 + 1];
        }
    }
    float qr[2], m2[2];
    {
        const float m2c = -2.f * csi[0];
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int64_t q = q0 + wq + i * 32 + l32;
            qr[i] = qn[q];
            m2[i] = m2c * qsi[q];
        }
    }
    cns[t_begin & 1][tid & (GT - 1)] = cn[(int64_t)tb * GT + (tid & (GT - 1))];
    __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));   // fragments and the first copies are in: the counts below start from an empty queue
    floatx16 acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;
    float *stage = stage_all + wave * (16 * SLD);

    // Writes out the minima collected for steps [t0, t1) (t1 - t0 <= BMC, t0 a multiple of BMC): for each
    // of the tile's 128 queries the 2 (t1 - t0) consecutive blocks starting at block 2 (tb + t0).  Four
    // lanes cover a row's 64 bytes, one store instruction 16 rows.  Every wavefront's minima of these
    // steps must be in LDS (a workgroup barrier lies between their epilogues and this call).
    const bool bm_vec = (nb & 3) == 0;                    // rows of bm start on 16-byte boundaries
    auto flush_bm = [&](int t0, int t1) {
        const int ncol = 2 * (t1 - t0);
        const int cq = (tid & 3) * 4;
#pragma unroll
        for (int pass = 0; pass < 2; ++pass) {
            const int row = pass * 64 + (tid >> 2);
            if (cq < ncol) {
                const float4 v = *reinterpret_cast<const float4 *>(&bmbuf[row * BMLD + cq]);
                float *dst = bm + (q0 + row) * (int64_t)nb + (int64_t)(tb + t0) * (GT / BMW) + cq;
                if (bm_vec && cq + 3 < ncol) {
                    *reinterpret_cast<float4 *>(dst) = v;
                } else {
                    const float e[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
                    for (int u = 0; u < 4; ++u)
                        if (cq + u < ncol) dst[u] = e[u];
                }
            }
        }
    };

    float cn_next = 0.f;
    for (int t = t_begin; t < t_end; ++t) {
        const int64_t c0 = (int64_t)(tb + t) * GT;
#pragma unroll
        for (int s = 0; s < STAGES; ++s) {
            // operations issued after the copy of this stage: the copies of the PD - 1 stages after it,
            // the norm load when it was issued in between, the epilogue stores when it lies in between
            // (the tile's one norm load is left out of the count: wherever the compiler places it,
            // waiting for one operation more than needed is harmless)
            constexpr int COPIES = 2 * (PD - 1);
            if (WHOLE) __builtin_amdgcn_s_waitcnt(vmcnt_imm(2 * STAGES - 2 + EPI_STORES));   // the same count at every step
            else if (s < PD) __builtin_amdgcn_s_waitcnt(vmcnt_imm(COPIES + EPI_STORES));
            else __builtin_amdgcn_s_waitcnt(vmcnt_imm(COPIES));
            asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
            if (!WHOLE) issue(t, s + PD);
            else if (s >= 1) issue(t, STAGES + s - 1);
            // the minima of the last BMC tiles are complete (every wavefront is past their epilogues)
            if (s == 0 && t > t_begin && (t - t_begin) % BMC == 0) flush_bm(t - t_begin - BMC, t - t_begin);
            // this tile's centroid norms, requested at the end of the previous tile (below), go to LDS
            // in the middle of this one: the stores of the previous epilogue and the copies of the
            // steps since were issued after that load
            if (s == STAGES / 2 && t > t_begin) {
                asm volatile("s_waitcnt vmcnt(%1)" : "+v"(cn_next) : "n"(EPI_STORES + 2 * (STAGES / 2)));
                cns[t & 1][tid & (GT - 1)] = cn_next;
            }
            // The centroid fragments are read with explicit instructions: for an ordinary LDS read of a
            // buffer that copies write, the compiler waits for every outstanding vector-memory
            // operation (the stores of the previous epilogue included).  The waits above and the
            // barrier already order these reads after the copy they need.
            const uint32_t bs = (uint32_t)reinterpret_cast<uintptr_t>(slot_of(s));   // LDS byte address
            gu32x4 b[2][2];
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                const int rb = wc + j * 32 + l32;
#pragma unroll
                for (int p = 0; p < 2; ++p) {
                    const uint32_t at = bs + 4u * (uint32_t)(rb * ROWF + (((2 * h + p) ^ ((rb >> 2) & 3)) << 2));
                    asm volatile("ds_read_b128 %0, %1" : "=v"(b[j][p]) : "v"(at));
                }
            }
            asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(b[0][0]), "+v"(b[0][1]), "+v"(b[1][0]), "+v"(b[1][1]));
#pragma unroll
            for (int e = 0; e < 3; ++e)
#pragma unroll
                for (int i = 0; i < 2; ++i)
#pragma unroll
                    for (int j = 0; j < 2; ++j) acc[i][j] = mfma3(b[j], afr[s][i], acc[i][j], e);
        }
        if (WHOLE) {   // everyone is done with the last buffer: refill it before the stores go out
            asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
            issue(t, 2 * STAGES - 1);
        }
        {   // norms of the next tile (index clamped past the end).  The load is hidden from the compiler,
            // which would otherwise drain the whole queue, stores included, where the value is used.
            // (cn_next's register is written when the load returns: nothing may read or move it before the
            // explicit wait at its use; the parity tests of this kernel are what checks a new build.)
            const int64_t cnx = c0 + GT + (tid & (GT - 1));
            const float *pn = cn + (cnx < K ? cnx : K - 1);
            asm volatile("global_load_dword %0, %1, off" : "=v"(cn_next) : "v"(pn) : "memory");
        }
        const float *cnw = cns[t & 1] + wc;
#pragma unroll
        for (int i = 0; i < 2; ++i)
            emit_block<false, EPI_SROWS, true>(acc[i], qr[i], m2[i], cnw, stage, q0 + wq + i * 32, nq, c0 + wc, K, Dt, ldt, bm, nb,
                                        &bmbuf[(wq + i * 32) * BMLD + ((t - t_begin) % BMC) * 2 + (wave & 1)], BMLD);
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int j = 0; j < 2; ++j)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;
    }
    __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));   // no copy into LDS may outlive the workgroup
    __syncthreads();                              // the last epilogues' minima are in LDS
    flush_bm((t_end - t_begin - 1) / BMC * BMC, t_end - t_begin);
}

// The same for small batches (latency mode): a workgroup takes 32 QT queries x 256 centroids (QT = 1
// or 2), all four wavefronts share the queries and each owns 64 of the centroids (2 QT
// accumulators), so a batch of up to 32 queries costs a quarter of the MFMA work of the
// 128-query tile and the kernel is bounded by streaming the centroid matrix once per batch of
// up to 64 queries.  Operand rows in LDS: the query rows, then 256 centroid rows per buffer,
// staged like the large tile.
constexpr int SKQ = 32, SKC = 256;

template <int QT>
__global__ __launch_bounds__(256) void coarse_gemm_skinny_kernel(
    const _Float16 *__restrict__ Qp, const float *__restrict__ qn, const float *__restrict__ qsi, int64_t nq,
    const _Float16 *__restrict__ Cp, const float *__restrict__ cn, const float *__restrict__ csi, int64_t K,
    int Dp, float *__restrict__ Dt, int64_t ldt, float *__restrict__ bm, int nb, int tiles_q)
{
    typedef const __attribute__((address_space(1))) void *gptr_t;
    typedef __attribute__((address_space(3))) void *lptr_t;
    static_assert(QT == 1 || QT == 2, "one or two blocks of 32 queries");
    constexpr int QROWS = QT * SKQ;
    constexpr int SKBUF = (QROWS + SKC) * ROWF;   // floats per operand buffer
    // two operand buffers, each reused as the output staging of two wavefronts
    constexpr int OPS = SKBUF > 2 * 32 * SLD ? SKBUF : 2 * 32 * SLD;
    __shared__ __attribute__((aligned(16))) float ops0[OPS];
    __shared__ __attribute__((aligned(16))) float ops1[OPS];
    __shared__ __attribute__((aligned(16))) float cns[SKC];
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    // The query tiles of one block of 256 centroids go to the same XCD (workgroup b runs on XCD b % 8),
    // one after the other: the centroid rows are fetched from HBM once and found in that XCD's L2 by
    // the other tiles.  Grid: 8 * ceil(blocks / 8) * tiles_q workgroups.
    const int64_t local = blockIdx.x / N_XCD;
    const int64_t cblk = (local / tiles_q) * N_XCD + blockIdx.x % N_XCD;
    const int64_t q0 = (local % tiles_q) * QROWS, c0 = cblk * SKC;
    if (c0 >= K) return;                                           // (before any barrier; uniform)
    const int wc = wave * 64;
    const int l32 = lane & 31, h = lane >> 5;
    cns[tid] = c0 + tid < K ? cn[c0 + tid] : 0.f;
    floatx16 acc[QT][2];
#pragma unroll
    for (int i = 0; i < QT; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;
    // Copies per stage: wave w takes the centroid blocks (16 rows each) w, w+4, w+8, w+12 with one
    // instruction in a rolled loop, the first 2 QT waves also one block of query rows (see gemm_tile).
    const int rl = lane >> 2;
    const int fq = (lane & 3) ^ ((rl >> 2) & 3);                       // (r >> 2) & 3 depends on the row inside the block only
    const float *srcc = reinterpret_cast<const float *>(Cp) + (c0 + wave * 16 + rl) * Dp + fq * 4;
    const float *srcq = reinterpret_cast<const float *>(Qp) + (q0 + (wave & (2 * QT - 1)) * 16 + rl) * Dp + fq * 4;
    auto issue = [&](int k0, float *dst) {
#pragma nounroll
        for (int n = 0; n < 4; ++n)
            __builtin_amdgcn_global_load_lds((gptr_t)(srcc + (int64_t)n * 64 * Dp + k0),
                                             (lptr_t)(dst + (2 * QT + wave + 4 * n) * 256), 16, 0, 0);
        if (wave < 2 * QT)
            __builtin_amdgcn_global_load_lds((gptr_t)(srcq + k0), (lptr_t)(dst + wave * 256), 16, 0, 0);
    };
    auto compute = [&](const float *As) {
        const float *Bs = As + QROWS * ROWF;
        gu32x4 a[QT][2], b[2][2];
#pragma unroll
        for (int i = 0; i < QT; ++i)
#pragma unroll
            for (int p = 0; p < 2; ++p)
                a[i][p] = *reinterpret_cast<const gu32x4 *>(&As[(i * 32 + l32) * ROWF + (((2 * h + p) ^ ((l32 >> 2) & 3)) << 2)]);
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const int rb = wc + j * 32 + l32;
#pragma unroll
            for (int p = 0; p < 2; ++p)
                b[j][p] = *reinterpret_cast<const gu32x4 *>(&Bs[rb * ROWF + (((2 * h + p) ^ ((rb >> 2) & 3)) << 2)]);
        }
#pragma unroll
        for (int e = 0; e < 3; ++e)
#pragma unroll
            for (int i = 0; i < QT; ++i)
#pragma unroll
                for (int j = 0; j < 2; ++j) acc[i][j] = mfma3(b[j], a[i], acc[i][j], e);
    };
    const int stages = Dp / DK;
    issue(0, ops0);
    for (int s = 0; s < stages; s += 2) {     // unrolled by two, see gemm_tile
        __builtin_amdgcn_s_waitcnt(0x0F70);
        __syncthreads();
        issue((s + 1) * DK, ops1);
        compute(ops0);
        __builtin_amdgcn_s_waitcnt(0x0F70);
        __syncthreads();
        if (s + 2 < stages) issue((s + 2) * DK, ops0);
        compute(ops1);
    }
    __syncthreads();
    const float m2c = -2.f * csi[0];
    float *stage = (wave < 2 ? ops0 : ops1) + (wave & 1) * (32 * SLD);
    const bool interior = q0 + QROWS <= nq && c0 + SKC <= K && (K & 3) == 0;
#pragma unroll
    for (int i = 0; i < QT; ++i) {
        const int64_t qb = q0 + i * 32, q = qb + l32;
        const float qr = q < nq ? qn[q] : 0.f;
        const float m2 = q < nq ? m2c * qsi[q] : 0.f;
        if (interior) emit_block<false>(acc[i], qr, m2, cns + wc, stage, qb, nq, c0 + wc, K, Dt, ldt, bm, nb);
        else emit_block<true>(acc[i], qr, m2, cns + wc, stage, qb, nq, c0 + wc, K, Dt, ldt, bm, nb);
    }
}

// Nearest centroid only (P = 1): the same tile product, reduced on the fly to
// the per-query minimum of (distance, centroid id), merged across centroid
// tiles with a 64-bit atomic minimum; no distance tile is written.  best[]
// must be pre-filled with all ones.
__global__ __launch_bounds__(256) void coarse_argmin_kernel(
    const _Float16 *__restrict__ Qp, const float *__restrict__ qn, const float *__restrict__ qsi, int64_t nq,
    const _Float16 *__restrict__ Cp, const float *__restrict__ cn, const float *__restrict__ csi, int64_t K,
    int Dp, unsigned long long *__restrict__ best, int tiles_q)
{
    __shared__ __attribute__((aligned(16))) float ops0[DBUF];
    __shared__ __attribute__((aligned(16))) float ops1[DBUF];
    __shared__ __attribute__((aligned(16))) float cns[GT];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    int64_t q0, c0;
    if (!tile_of_block(blockIdx.x, tiles_q, q0, c0)) return;
    const int wq = (wave >> 1) * 64, wc = (wave & 1) * 64;
    const int l32 = lane & 31, h = lane >> 5;
    if (threadIdx.x < GT) cns[threadIdx.x] = c0 + threadIdx.x < K ? cn[c0 + threadIdx.x] : 0.f;
    floatx16 acc[2][2];
    gemm_tile(Qp, nq, q0, Cp, K, c0, Dp, ops0, ops1, acc);
    const float m2c = -2.f * csi[0];
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int64_t q = q0 + wq + i * 32 + l32;
        const float qr = q < nq ? qn[q] : 0.f;
        const float m2 = q < nq ? m2c * qsi[q] : 0.f;
        unsigned long long key = ~0ull;
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int cl = wc + j * 32 + 8 * (v >> 2) + 4 * h + (v & 3);
                const int64_t c = c0 + cl;
                if (c < K) {
                    float d = fmaxf(fmaf(m2, acc[i][j][v], qr + cns[cl]), 0.f);
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

// ---- Nearest centroid through a certified shortlist ----
// The hi halves alone give <q,c> to about 2^-10 of |q||c| at a third of the MFMA work.  With
//   approx(q,c) = |q|^2 + |c|^2 - 2 <hi(q), hi(c)>  (fp32 accumulation),
//   eps(q,c)    = 2^-9 (|q|^2 + |c|^2) + abs_term,
// the exact squared distance d lies in [approx - eps, approx + eps]: an element of hi(x) differs from x
// by at most 2^-11 |x_i| (fp16 rounding; below the normal range by at most 2^-39 of the largest
// magnitude under the row's or table's scale, which abs_term covers), so the inner product is off by at
// most (2^-10 + 2^-22) sum |q_i c_i| <= (2^-11 + 2^-23)(|q|^2 + |c|^2), the distance by twice that,
// and the factor 2^-9 leaves as much again for the fp32 roundings of the accumulation and the epilogue.
// U[q], the smallest approx + eps seen so far, never drops below the true minimum distance of q, so
// every centroid that attains that minimum has approx - eps <= U[q] whenever it is looked at: the
// kernel appends each (q, c) with approx - eps <= U[q] to a candidate list, and rerank_kernel decides
// among the candidates with exact arithmetic.  Stale reads of U only lengthen the list.

// Row r of the hi-only table from row r of the hi/lo table (split_rows_kernel; Dp dimensions, a multiple
// of 32): per 32 dimensions the 16-byte chunks [k 0-7 | k 16-23 | k 8-15 | k 24-31], so that lane half h
// of gemm_tile<true> finds its dimensions of the two 16-wide products in chunks 2h and 2h+1.
__global__ __launch_bounds__(256) void pack_hi_kernel(const _Float16 *__restrict__ P, int64_t n_rows, int Dp,
                                                      _Float16 *__restrict__ H)
{
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;   // one 16-byte chunk of the output each
    const int chunks = Dp / 8;
    if (i >= n_rows * chunks) return;
    const int64_t r = i / chunks;
    const int ch = (int)(i % chunks), t = ch >> 2, slot = ch & 3;
    const int k8 = (slot & 1) * 2 + (slot >> 1);               // which 8 dimensions of the 32: slots 0,1,2,3 -> 0,2,1,3
    const int dim = 32 * t + 8 * k8;                            // first dimension of the chunk
    // in the hi/lo table dimension d sits at stage d / 16: [hi k0..7 | lo k0..7 | hi k8..15 | lo k8..15]
    const _Float16 *src = P + r * (int64_t)Dp * 2 + (dim >> 4) * 32 + ((dim >> 3) & 1) * 16;
    *reinterpret_cast<gu32x4 *>(H + r * (int64_t)Dp + ch * 8) = *reinterpret_cast<const gu32x4 *>(src);
}

constexpr float SHORTLIST_KAPPA = 0x1p-9f;
constexpr int SHORTLIST_SEGS = 64;

// gmax_bits: the centroid table's largest magnitude (bit pattern), D: the dimension; abs_term =
// 2^-30 (|q|^2 + D gmax^2) covers what lies below fp16's normal range under the table-wide scale.
// U must be pre-filled with all ones, the segment counters with 0; pairs beyond a segment's capacity are
// dropped (the caller compares the counters with seg_cap and falls back to the exact kernel).
__global__ __launch_bounds__(256) void coarse_shortlist_kernel(
    const _Float16 *__restrict__ Qh, const float *__restrict__ qn, const float *__restrict__ qsi, int64_t nq,
    const _Float16 *__restrict__ Ch, const float *__restrict__ cn, const float *__restrict__ csi, int64_t K,
    int Dph, int D, uint32_t *__restrict__ U, int2 *__restrict__ cand_all, unsigned long long *__restrict__ cand_count_all,
    unsigned long long seg_cap, int tiles_q)
{
    // the list is kept in SHORTLIST_SEGS segments with a counter each (128 bytes apart), so that the appends
    // of different workgroups do not all queue at one address
    int2 *cand = cand_all + (blockIdx.x % SHORTLIST_SEGS) * seg_cap;
    unsigned long long *cand_count = cand_count_all + (blockIdx.x % SHORTLIST_SEGS) * 16;
    const unsigned long long cand_cap = seg_cap;
    __shared__ __attribute__((aligned(16))) float ops0[DBUF];
    __shared__ __attribute__((aligned(16))) float ops1[DBUF];
    __shared__ __attribute__((aligned(16))) float cns[GT];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    int64_t q0, c0;
    if (!tile_of_block(blockIdx.x, tiles_q, q0, c0)) return;
    const int wq = (wave >> 1) * 64, wc = (wave & 1) * 64;
    const int l32 = lane & 31, h = lane >> 5;
    if (threadIdx.x < GT) cns[threadIdx.x] = c0 + threadIdx.x < K ? cn[c0 + threadIdx.x] : 0.f;
    // the bounds as they stand now, requested before the product so that their latency is hidden under it
    // (an older bound is a weaker one, never a wrong one)
    uint32_t seen[2];
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int64_t q = q0 + wq + i * 32 + l32;
        seen[i] = q < nq ? __hip_atomic_load(&U[q], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : 0u;
    }
    floatx16 acc[2][2];
    gemm_tile<true>(Qh, nq, q0, Ch, K, c0, Dph, ops0, ops1, acc);
    const float m2c = -2.f * csi[0];
    const float gmax = __uint_as_float(reinterpret_cast<const uint32_t *>(csi)[1]);
    const float abs_c = 0x1p-30f * (float)D * gmax * gmax;
    const bool whole = c0 + GT <= K;                     // no centroid of the tile lies past the end
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int64_t q = q0 + wq + i * 32 + l32;
        const bool qok = q < nq;
        const float qr = qok ? qn[q] : 0.f;
        const float m2 = qok ? m2c * qsi[q] : 0.f;
        const float abs_term = fmaf(0x1p-30f, qr, abs_c);
        // t[j][g] = |q|^2 + |c|^2 of the lane's four consecutive centroids 32 j + 8 g + 4 h ..
        float4 t[2][4];
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const float4 cv = *reinterpret_cast<const float4 *>(&cns[wc + j * 32 + 8 * g + 4 * h]);
                t[j][g] = make_float4(qr + cv.x, qr + cv.y, qr + cv.z, qr + cv.w);
            }
        // upper ends first: this block's smallest approx + eps joins the bound before anything is kept
        float umin = INFINITY;
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const float tv[4] = {t[j][g].x, t[j][g].y, t[j][g].z, t[j][g].w};
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const float up = fmaf(m2, acc[i][j][4 * g + r], fmaf(SHORTLIST_KAPPA, tv[r], tv[r]));
                    if (whole || c0 + wc + j * 32 + 8 * g + 4 * h + r < K) umin = fminf(umin, up);
                }
            }
        umin = fmaxf(umin + abs_term, 0.f);
        umin = fminf(umin, __shfl_xor(umin, 32, WAVE));
        if (!qok) continue;
        float bound = umin;
        if (seen[i] != ~0u) bound = fminf(bound, __uint_as_float(seen[i]));
        // (non-negative floats order like their bit patterns)
        if (h == 0 && __float_as_uint(umin) < seen[i]) atomicMin(&U[q], __float_as_uint(umin));
        bound += abs_term;   // lo = approx - eps <= bound  <=>  approx - kappa t <= bound + abs_term
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const float tv[4] = {t[j][g].x, t[j][g].y, t[j][g].z, t[j][g].w};
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const float lo = fmaf(m2, acc[i][j][4 * g + r], fmaf(-SHORTLIST_KAPPA, tv[r], tv[r]));
                    const int cl = wc + j * 32 + 8 * g + 4 * h + r;
                    if (lo <= bound && (whole || c0 + cl < K)) {
                        const unsigned long long at = atomicAdd(cand_count, 1ull);
                        if (at < cand_cap) cand[at] = make_int2((int)q, (int)(c0 + cl));
                    }
                }
            }
    }
}

// The same pass with the structure of the sweep kernel, for SH = 3 or 4 hi-only stages (packed dimension
// 96 or 128): a workgroup keeps the hi fragments of ONE query tile in registers and sweeps `tiles_per_wg`
// consecutive centroid tiles through two LDS buffers of a whole tile each, one workgroup barrier per tile
// (the copies of tile t + 1 are issued right behind the barrier of tile t and waited for at the barrier of
// tile t + 1).  The running minimum of approx + eps over the sweep stays in registers and reaches U[q]
// once, at the end.
// Only direct-to-LDS copies write `ring` and `cns`, only explicit ds_read instructions read them.
template <int SH>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(SH == 3 ? 3 : 2, SH == 3 ? 3 : 2))) void coarse_shortlist_sweep_kernel(
    const _Float16 *__restrict__ Qh, const float *__restrict__ qn, const float *__restrict__ qsi, int64_t nq,
    const _Float16 *__restrict__ Ch, const float *__restrict__ cn, const float *__restrict__ csi, int64_t K,
    int D, uint32_t *__restrict__ U, int2 *__restrict__ cand_all, unsigned long long *__restrict__ cand_count_all,
    unsigned long long seg_cap, int tiles_q, int tiles_c, int tiles_per_wg)
{
    typedef const __attribute__((address_space(1))) void *gptr_t;
    typedef __attribute__((address_space(3))) void *lptr_t;
    constexpr int Dpf = SH * DK;                           // floats per row of the hi-only tables
    constexpr int SLOT = GT * ROWF;
    __shared__ __attribute__((aligned(16))) float ring[2][SH * SLOT];
    __shared__ __attribute__((aligned(16))) float cns[2][GT];
    int2 *cand = cand_all + (blockIdx.x % SHORTLIST_SEGS) * seg_cap;
    unsigned long long *cand_count = cand_count_all + (blockIdx.x % SHORTLIST_SEGS) * 16;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l32 = lane & 31, h = lane >> 5;
    const int wq = (wave >> 1) * 64, wc = (wave & 1) * 64;
    const int tq_per = (tiles_q + N_XCD - 1) / N_XCD;
    const int xcd = (int)(blockIdx.x % N_XCD);
    const int64_t local = blockIdx.x / N_XCD;
    const int tq = (int)(local % tq_per) * N_XCD + xcd;
    if (tq >= tiles_q) return;
    const int tb = (int)(local / tq_per) * tiles_per_wg;
    int t_end = tb < tiles_c ? tiles_c - tb : 0;
    if (t_end > tiles_per_wg) t_end = tiles_per_wg;
    if (t_end <= 0) return;
    const int64_t q0 = (int64_t)tq * GT;

    // this wavefront's copies of a tile: rows 32 wave + 16 n + lane / 4 (n = 0, 1) of each stage, and
    // (wavefronts 0, 1) 64 of the tile's norms (index clamped at the end of the table: never used there)
    const int rl = wave * 32 + (lane >> 2);
    const int fl = (lane & 3) ^ ((lane >> 4) & 3);
    const float *cbase = reinterpret_cast<const float *>(Ch) + (int64_t)rl * Dpf + fl * 4;
    auto issue_tile = [&](int t) {
        const int tc = t < t_end ? t : t_end - 1;            // past the range: the last tile again, never read
        if (wave < 2) {
            const int64_t cnx = (int64_t)(tb + tc) * GT + wave * 64 + lane;
            __builtin_amdgcn_global_load_lds((gptr_t)(cn + (cnx < K ? cnx : K - 1)), (lptr_t)(&cns[t & 1][wave * 64]), 4, 0, 0);
        }
        const float *src = cbase + (int64_t)(tb + tc) * GT * Dpf;
        float *dst = &ring[t & 1][wave * 512];
        // (one instruction in a rolled loop: the compiler tracks only a handful of distinct LDS copies exactly)
#pragma nounroll
        for (int n = 0; n < 2 * SH; ++n)
            __builtin_amdgcn_global_load_lds((gptr_t)(src + (n >> 1) * DK + (int64_t)(n & 1) * 16 * Dpf),
                                             (lptr_t)(dst + (n >> 1) * SLOT + (n & 1) * 256), 16, 0, 0);
    };
    issue_tile(0);

    gu32x4 afr[SH][2][2];
    float qr[2], m2[2], abs_term[2], lmin[2];
    uint32_t seen[2];
    bool qok[2];
    {
        const float m2c = -2.f * csi[0];
        const float gmax = __uint_as_float(reinterpret_cast<const uint32_t *>(csi)[1]);
        const float abs_c = 0x1p-30f * (float)D * gmax * gmax;
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int64_t q = q0 + wq + i * 32 + l32;
            qok[i] = q < nq;
            const gu32x4 *row = reinterpret_cast<const gu32x4 *>(reinterpret_cast<const float *>(Qh) + q * Dpf) + 2 * h;
#pragma unroll
            for (int s = 0; s < SH; ++s) {
                afr[s][i][0] = row[s * 4 + 0];
                afr[s][i][1] = row[s * 4 + 1];
            }
            qr[i] = qok[i] ? qn[q] : 0.f;
            m2[i] = qok[i] ? m2c * qsi[q] : 0.f;
            abs_term[i] = fmaf(0x1p-30f, qr[i], abs_c);
            // the bound as it stands now (an older bound is a weaker one, never a wrong one)
            seen[i] = qok[i] ? __hip_atomic_load(&U[q], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : 0u;
            lmin[i] = INFINITY;
        }
    }

    for (int t = 0; t < t_end; ++t) {
        __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));   // this wavefront's copies of tile t (issued a tile ago) are in
        asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");   // ... and everyone's; tile t - 1's buffer is free
        issue_tile(t + 1);
        const int64_t c0 = (int64_t)(tb + t) * GT;
        const bool whole = c0 + GT <= K;
        // One half of the wavefront's 64 centroids at a time, both blocks of 32 queries: two accumulators live
        // instead of four, every centroid fragment still read from LDS once.  Registers are what limits the
        // wavefronts per SIMD here, and three of them hide the LDS and barrier latencies that two leave open.
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            floatx16 acc[2];
            const int rb = wc + j * 32 + l32;
#pragma unroll
            for (int s = 0; s < SH; ++s) {
                gu32x4 b[2];
                const uint32_t bs = (uint32_t)reinterpret_cast<uintptr_t>(&ring[t & 1][s * SLOT]);
#pragma unroll
                for (int p = 0; p < 2; ++p) {
                    const uint32_t at = bs + 4u * (uint32_t)(rb * ROWF + (((2 * h + p) ^ ((rb >> 2) & 3)) << 2));
                    asm volatile("ds_read_b128 %0, %1" : "=v"(b[p]) : "v"(at));
                }
                asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(b[0]), "+v"(b[1]));
#pragma unroll
                for (int p = 0; p < 2; ++p)
#pragma unroll
                    for (int i = 0; i < 2; ++i) {
                        floatx16 c_in = acc[i];
                        if (s == 0 && p == 0) {
#pragma unroll
                            for (int v = 0; v < 16; ++v) c_in[v] = 0.f;
                        }
                        acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(halfx8, b[p]),
                                                                        __builtin_bit_cast(halfx8, afr[s][i][p]), c_in, 0, 0, 0);
                    }
            }
            // the norms of the lane's 16 centroids of this half (copied to LDS behind the compiler's back:
            // explicit reads and wait)
            floatx4 cv[4];
            {
                const uint32_t cb = (uint32_t)reinterpret_cast<uintptr_t>(&cns[t & 1][wc + j * 32 + 4 * h]);
#pragma unroll
                for (int g = 0; g < 4; ++g) asm volatile("ds_read_b128 %0, %1" : "=v"(cv[g]) : "v"(cb + 32u * (uint32_t)g));
                asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(cv[0]), "+v"(cv[1]), "+v"(cv[2]), "+v"(cv[3]));
            }
            uint32_t valid = 0xFFFFu;                          // bit v: the lane's centroid v lies inside the table
            if (!whole) {
                valid = 0;
#pragma unroll
                for (int v = 0; v < 16; ++v) valid |= (c0 + wc + j * 32 + 8 * (v >> 2) + 4 * h + (v & 3) < K ? 1u : 0u) << v;
            }
            const float cmax = fmaxf(fmaxf(fmaxf(fmaxf(cv[0][0], cv[0][1]), fmaxf(cv[0][2], cv[0][3])), fmaxf(fmaxf(cv[1][0], cv[1][1]), fmaxf(cv[1][2], cv[1][3]))),
                                     fmaxf(fmaxf(fmaxf(cv[2][0], cv[2][1]), fmaxf(cv[2][2], cv[2][3])), fmaxf(fmaxf(cv[3][0], cv[3][1]), fmaxf(cv[3][2], cv[3][3]))));
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                // a = approx, in place, and its minimum over the lane's centroids: with their largest
                // t = |q|^2 + |c|^2, three operations per distance decide, nearly always, that the lane has
                // nothing to report
                float amin = INFINITY;
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const float a = fmaf(m2[i], acc[i][v], qr[i] + cv[v >> 2][v & 3]);
                    acc[i][v] = a;
                    if (whole || (valid >> v & 1)) amin = fminf(amin, a);
                }
                float bound = lmin[i];
                if (seen[i] != ~0u) bound = fminf(bound, __uint_as_float(seen[i]));
                // every lower end of the lane is at least amin - kappa tmax - abs_term, every upper end at least
                // amin: above the bound, the lane can neither list a centroid nor lower the bound
                const bool look = fmaf(-SHORTLIST_KAPPA, qr[i] + cmax, amin) - abs_term[i] <= bound;
                if (__any(look)) {
                    // the smallest upper end a + kappa t + abs_term of the query in this half, exactly
                    float umin = INFINITY;
#pragma unroll
                    for (int v = 0; v < 16; ++v) {
                        const float up = fmaf(SHORTLIST_KAPPA, qr[i] + cv[v >> 2][v & 3], acc[i][v]);
                        if (whole || (valid >> v & 1)) umin = fminf(umin, up);
                    }
                    umin = fmaxf(umin + abs_term[i], 0.f);
                    umin = fminf(umin, __shfl_xor(umin, 32, WAVE));   // the other lane half holds the other 16 centroids
                    lmin[i] = fminf(lmin[i], umin);
                    bound = fminf(bound, lmin[i]) + abs_term[i];   // approx - eps <= bound  <=>  a - kappa t <= bound + abs_term
                    uint32_t todo = 0;                                // which of the lane's distances pass
#pragma unroll
                    for (int v = 0; v < 16; ++v)
                        todo |= (fmaf(-SHORTLIST_KAPPA, qr[i] + cv[v >> 2][v & 3], acc[i][v]) <= bound ? 1u : 0u) << v;
                    todo &= valid;
                    if (!qok[i]) todo = 0;
                    while (todo) {
                        const int v = __builtin_ctz(todo);
                        todo &= todo - 1;
                        const unsigned long long at = atomicAdd(cand_count, 1ull);
                        if (at < seg_cap)
                            cand[at] = make_int2((int)(q0 + wq + i * 32 + l32), (int)(c0 + wc + j * 32 + 8 * (v >> 2) + 4 * h + (v & 3)));
                    }
                }
            }
            __builtin_amdgcn_sched_barrier(0);   // the next half's products start with this half's registers free
        }
    }
    __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));   // no copy into LDS may outlive the workgroup
#pragma unroll
    for (int i = 0; i < 2; ++i)   // (non-negative floats order like their bit patterns)
        if (qok[i] && h == 0 && __float_as_uint(lmin[i]) < seen[i]) atomicMin(&U[q0 + wq + i * 32 + l32], __float_as_uint(lmin[i]));
}

// Exact decision among the candidates: one wavefront per pair computes |x - c|^2 from the fp32 rows
// (differences squared, summed in a tree over the lanes: a few ulps) and merges (distance, id) into
// best[q] with a 64-bit atomic minimum.  best must be pre-filled with all ones.
// Grid: (quarter of the longest segment, SHORTLIST_SEGS).
__global__ __launch_bounds__(256) void rerank_kernel(const float *__restrict__ X, const float *__restrict__ C, int D,
                                                     const int2 *__restrict__ cand_all, const unsigned long long *__restrict__ cand_count_all,
                                                     unsigned long long seg_cap, unsigned long long *__restrict__ best)
{
    const int64_t i = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    const int lane = threadIdx.x & 63;
    if ((unsigned long long)i >= cand_count_all[blockIdx.y * 16]) return;
    const int2 qc = cand_all[blockIdx.y * seg_cap + i];
    const float *x = X + (int64_t)qc.x * D, *c = C + (int64_t)qc.y * D;
    float s = 0.f;
    for (int k = lane; k < D; k += WAVE) {
        const float u = x[k] - c[k];
        s = fmaf(u, u, s);
    }
    s = wave_sum(s);
    if (lane == 0) atomicMin(&best[qc.x], ((unsigned long long)float_key(s) << 32) | (uint32_t)qc.y);
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
__global__ __launch_bounds__(BLOCK) void probe_select_kernel(const float *__restrict__ Dt, int64_t ldt,
                                                             const float *__restrict__ bm, int64_t K,
                                                             int nb, int P,
                                                             int32_t *__restrict__ probe_id,
                                                             float *__restrict__ probe_d)
{
    __shared__ SelectShared sh;
    __shared__ uint32_t nflag_s;
    extern __shared__ int blist[];
    const int64_t q = blockIdx.x;
    const float *row = Dt + q * ldt;
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

// The same selection with the keys held in LDS, for nb <= PS_NB_MAX block minima and
// P <= PS_P_MAX: the block minima are read once (not once per radix pass), and of the flagged
// blocks' elements only those at or below the block threshold t are kept (t is the P-th
// smallest block minimum, so the P closest centroids are among them; with randomly numbered
// centroids little more than P survive), compacted in ascending centroid id, and selected
// from LDS.  A query with more than PS_CAP survivors (duplicated centroids) takes the
// global-memory path of probe_select_kernel.  Dynamic LDS: 2P + 3 + max(nb, 2 PS_CAP) words.
constexpr int PS_NB_MAX = 16384, PS_P_MAX = 256, PS_CAP = 4096;

// (the body, for query q of the batch: also the first half of select_score_prune_kernel)
__device__ __forceinline__ void probe_select_lds_body(const float *__restrict__ Dt, int64_t ldt,
                                                      const float *__restrict__ bm, int64_t K, int nb, int P,
                                                      int32_t *__restrict__ probe_id, float *__restrict__ probe_d,
                                                      int64_t q, int *ps_dyn)
{
    constexpr int BLOCK = 1024;
    __shared__ SelectShared sh;
    __shared__ uint32_t nflag_s;
    int *blist = ps_dyn;                                           // 2P flagged blocks
    uint32_t *keys = reinterpret_cast<uint32_t *>(ps_dyn + ((2 * P + 3) & ~3));   // (16-byte aligned) nb block-minimum keys, then the survivors
    const int tid = threadIdx.x;
    const float *row = Dt + q * ldt;
    const float *bmr = bm + q * nb;
    if ((nb & 3) == 0) {   // rows of bm are then 16-byte aligned: four loads in flight per thread, 128 bits each
        const float4 *src = reinterpret_cast<const float4 *>(bmr);
        for (int i0 = tid; i0 < nb / 4; i0 += 4 * BLOCK) {
            float4 v[4];
#pragma unroll
            for (int u = 0; u < 4; ++u)
                if (i0 + u * BLOCK < nb / 4) v[u] = src[i0 + u * BLOCK];
#pragma unroll
            for (int u = 0; u < 4; ++u)
                if (i0 + u * BLOCK < nb / 4)
                    *reinterpret_cast<uint4 *>(&keys[4 * (i0 + u * BLOCK)]) =
                        make_uint4(float_key(v[u].x), float_key(v[u].y), float_key(v[u].z), float_key(v[u].w));
        }
    } else {
        for (int i = tid; i < nb; i += BLOCK) keys[i] = float_key(bmr[i]);
    }
    __syncthreads();
    auto keyb = [keys](int64_t b) { return keys[b]; };
    const uint32_t nselb = P < nb ? (uint32_t)P : (uint32_t)nb;
    uint32_t t, needb;
    block_radix_select<BLOCK>(keyb, nb, nselb, sh, t, needb);
    static_assert(PS_NB_MAX <= 16 * BLOCK && PS_CAP <= 4 * BLOCK, "items per thread of the two ordered emits below");
    uint32_t nflag = block_emit_selected_runs<BLOCK, 4>(keys, nb, t, (uint32_t)P, sh,
                                                     [&](uint32_t pos, int64_t b, uint32_t) { blist[pos] = (int)b; });
    if (tid == 0) nflag_s = nflag;
    __syncthreads();                                               // blist complete, the block keys are dead
    nflag = nflag_s;
    const uint32_t tf = nb >= P ? t : 0xFFFFFFFFu;                 // fewer blocks than P: no filter
    // Candidates: the 64 distances of every flagged block, a block per wavefront and step (one
    // 256-byte row piece per load instruction), 16 blocks in flight per wavefront.  Survivors (at or
    // below the block threshold) are compacted in ascending centroid id: inside a wavefront by
    // ballots, across wavefronts by one workgroup scan of the wavefronts' counts per round.
    constexpr int CB = 16;                                         // blocks per wavefront and round
    const int wave = tid >> 6, lane = tid & 63;
    uint32_t *sk = keys;
    int *si = reinterpret_cast<int *>(keys + PS_CAP);
    uint32_t total = 0;                                            // survivors so far
    bool overflow = false;
    for (int b0 = 0; b0 < (int)nflag; b0 += CB * (BLOCK / WAVE)) { // uniform
        uint32_t kv[CB];
#pragma unroll
        for (int j = 0; j < CB; ++j) {
            const int bi = b0 + wave * CB + j;
            uint32_t k = 0xFFFFFFFFu;
            if (bi < (int)nflag) {
                const int64_t c = (int64_t)blist[bi] * BMW + lane;
                if (c < K) k = float_key(row[c]);
            }
            kv[j] = k;
        }
        uint32_t wcnt = 0;
#pragma unroll
        for (int j = 0; j < CB; ++j) wcnt += (uint32_t)__popcll(__ballot(kv[j] <= tf && kv[j] != 0xFFFFFFFFu));
        uint32_t round_total;
        const uint32_t exc = block_exclusive_scan<BLOCK>(lane == 0 ? wcnt : 0u, sh.scan, round_total);
        if (total + round_total > (uint32_t)PS_CAP) { overflow = true; break; }   // uniform
        uint32_t at = total + (uint32_t)__builtin_amdgcn_readfirstlane((int)exc);   // the wavefront's next output slot
#pragma unroll
        for (int j = 0; j < CB; ++j) {
            const bool sel = kv[j] <= tf && kv[j] != 0xFFFFFFFFu;
            const uint64_t m = __ballot(sel);
            if (sel) {
                const uint32_t o = at + __builtin_amdgcn_mbcnt_hi((uint32_t)(m >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)m, 0u));
                sk[o] = kv[j];
                si[o] = blist[b0 + wave * CB + j] * BMW + lane;
            }
            at += (uint32_t)__popcll(m);
        }
        total += round_total;
    }
    if (overflow || total < (uint32_t)P) {                          // uniform; the second cannot happen for nb >= P
        const int n_c = (int)nflag * BMW;
        __syncthreads();
        auto key = [&](int64_t v) {
            const int64_t c = (int64_t)blist[v >> 6] * BMW + (v & 63);
            return c < K ? float_key(row[c]) : 0xFFFFFFFFu;
        };
        uint32_t pivot, need;
        block_radix_select<BLOCK>(key, (int64_t)n_c, (uint32_t)P, sh, pivot, need);
        block_emit_selected<BLOCK>(key, (int64_t)n_c, (uint32_t)P, pivot, need, sh,
                                   [&](uint32_t pos, int64_t v, uint32_t k) {
                                       probe_id[q * P + pos] = blist[v >> 6] * BMW + (int)(v & 63);
                                       probe_d[q * P + pos] = key_float(k);
                                   });
        return;
    }
    __syncthreads();
    auto skey = [sk](int64_t i) { return sk[i]; };
    uint32_t pivot, need;
    block_radix_select<BLOCK>(skey, (int64_t)total, (uint32_t)P, sh, pivot, need);
    block_emit_selected_runs<BLOCK, 1>(sk, (int)total, pivot, need, sh,
                                    [&](uint32_t pos, int64_t i, uint32_t k) {
                                        probe_id[q * P + pos] = si[i];
                                        probe_d[q * P + pos] = key_float(k);
                                    });
}

__global__ __launch_bounds__(1024) __attribute__((amdgpu_waves_per_eu(8, 8))) void probe_select_lds_kernel(const float *__restrict__ Dt, int64_t ldt,
                                                                const float *__restrict__ bm, int64_t K,
                                                                int nb, int P,
                                                                int32_t *__restrict__ probe_id,
                                                                float *__restrict__ probe_d)
{
    extern __shared__ __attribute__((aligned(16))) int ps_dyn[];
    probe_select_lds_body(Dt, ldt, bm, K, nb, P, probe_id, probe_d, blockIdx.x, ps_dyn);
}

}  // namespace ivf
