// Stages 2-4 of the query path: subcentroid scoring by the closed form of
// Eq. (7), pruning to the S closest subregions, and the per-query table of
// -2<q_m, r^m_j> of Eq. (6).
#pragma once
#include "select.hpp"

namespace ivf {

// One kept subregion of one query, as the scan consumes it.
struct SubDesc {
    uint32_t blk;    // start of the subregion's record block, in BLK_ALIGN-byte units
    uint32_t pos0;   // grouped position of its first point (indexes ids[])
    uint32_t len;    // number of points
    float base;      // distance from the query to the subcentroid
};

// T[q][m][j] = -2 <q_m, r^m_j> (Eq. (6)) for one query by one workgroup of BLOCK threads: the query
// in LDS (qs, D floats), every thread one (sub-quantiser, codeword) pair at a time, each entry one
// chain of fused multiply-adds over the block's dimensions.
template <int BLOCK>
__device__ __forceinline__ void lut_body(const float *__restrict__ Qrow, int D, int M,
                                         const float *__restrict__ codebook, float *__restrict__ Tq, float *qs)
{
    const int ds = D / M;
    for (int i = threadIdx.x; i < D; i += BLOCK) qs[i] = Qrow[i];
    __syncthreads();
    for (int e = threadIdx.x; e < M * 256; e += BLOCK) {
        const int m = e >> 8;
        const float *cw = codebook + (int64_t)e * ds;
        float s = 0.f;
        for (int i = 0; i < ds; ++i) s = fmaf(qs[m * ds + i], cw[i], s);
        Tq[e] = -2.f * s;
    }
}

// Stages 2 and 3 fused, one workgroup per query.
// Stage 2 (Eq. (7)): score[p][l] = (1-a) D[q][r] + a D[q][nbr[r][l]] + cst[r][l], r = probe_id[q][p],
// cst[r][l] = -a(1-a)||c_r - s_l||^2 tabulated at load time.  The neighbour distances are gathered from
// the stage-1 distance tile, not recomputed; every thread has PL/BLOCK independent gathers in flight.
// The scores never leave the chip: they are kept in LDS as order-preserving keys.
// Stage 3: keep the S smallest of the P*L scores by (score, r*L + l).  probe_id is ascending in r, so
// position order in the score row is subregion-id order and the descriptors come out sorted by address.
// The selection leaves the kept score indices, in order, in LDS (over the keys, which every thread
// holds in registers by then) and their scores in the descriptors; the rest of a descriptor is
// then filled position by position, consecutive lanes writing consecutive descriptors, with the
// reads of the subregion table of four positions in flight per thread (filled item by item as
// they were selected, every read of that table was waited for before the next was issued).
// Dynamic LDS: P*L keys + P probe ids + P probe distances + P alphas.  P*L <= 4 * MAXV * BLOCK.
// Stage 4 rides along: the grid has 2 nq workgroups, and workgroup nq + q builds query q's lookup
// table (lut_body, from Qt = the queries, rotated if the index has a rotation) while the first nq
// gather and select; the two halves share nothing, and the table work hides under the gathers.
// Dynamic LDS must also hold D floats.
// (the body of a scoring workgroup, for query q of the batch: also the second half of select_score_prune_kernel)
template <int BLOCK, int MAXV>
__device__ __forceinline__ void score_prune_body(
    const float *__restrict__ Dt, int64_t ldt, int64_t K, const int32_t *__restrict__ probe_id,
    const float *__restrict__ probe_d, int P, int L, const int32_t *__restrict__ nbr,
    const float *__restrict__ cst, const float *__restrict__ alpha, int S,
    const uint4 *__restrict__ sub_info,
    SubDesc *__restrict__ desc, int64_t *__restrict__ kept_sub, int64_t *__restrict__ n_scanned,
    int64_t q, uint32_t *dyn)
{
    __shared__ SelectShared sh;
    __shared__ unsigned long long codes_total;
    const int PL = P * L;
    uint32_t *keys = dyn;
    int32_t *pid = reinterpret_cast<int32_t *>(dyn + PL);
    float *pd = reinterpret_cast<float *>(dyn + PL + P);
    float *pa = reinterpret_cast<float *>(dyn + PL + 2 * P);
    const float *row = Dt + q * ldt;
    for (int p = threadIdx.x; p < P; p += BLOCK) {
        const int32_t r = probe_id[q * P + p];
        pid[p] = r;
        pd[p] = probe_d[q * P + p];
        pa[p] = alpha[r];
    }
    if (threadIdx.x == 0) codes_total = 0;
    __syncthreads();
#pragma unroll 4
    for (int i = threadIdx.x; i < PL; i += BLOCK) {
        const int p = i / L, l = i - p * L;
        const int64_t r = pid[p];
        const float a = pa[p];
        const float ds = row[nbr[r * L + l]];
        keys[i] = float_key(fmaf(a, ds, fmaf(1.f - a, pd[p], cst[r * L + l])));
    }
    __syncthreads();
    auto key = [keys](int64_t i) { return keys[i]; };
    uint32_t pivot, need;
    block_radix_select<BLOCK>(key, PL, (uint32_t)S, sh, pivot, need);
    float *base_of = &desc[q * S].base;                  // stride of one descriptor: 4 floats
    block_emit_selected_runs<BLOCK, MAXV>(keys, PL, pivot, need, sh,
                                          [&](uint32_t pos, int64_t i, uint32_t k) {
                                              keys[pos] = (uint32_t)i;
                                              base_of[4 * pos] = key_float(k);
                                          });
    __syncthreads();
    unsigned long long mine = 0;
    for (int p0 = 0; p0 < S; p0 += 4 * BLOCK) {
        uint4 info[4];
        int64_t sub[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int pos = p0 + u * BLOCK + (int)threadIdx.x;
            if (pos < S) {
                const int i = (int)keys[pos];
                sub[u] = (int64_t)pid[i / L] * L + (i % L);
                info[u] = sub_info[sub[u]];                // one 16-byte read per kept subregion
            }
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int pos = p0 + u * BLOCK + (int)threadIdx.x;
            if (pos < S) {
                uint32_t *d = &desc[q * S + pos].blk;      // blk, pos0, len: the first 12 bytes
                d[0] = info[u].x;
                d[1] = info[u].y;
                d[2] = info[u].z;
                if (kept_sub) kept_sub[q * S + pos] = sub[u];
                mine += info[u].z;
            }
        }
    }
    if (mine) atomicAdd(&codes_total, mine);
    __syncthreads();
    if (threadIdx.x == 0 && n_scanned) n_scanned[q] = (int64_t)codes_total;
}

template <int BLOCK, int MAXV>
__global__ __launch_bounds__(BLOCK) void score_prune_kernel(
    const float *__restrict__ Dt, int64_t ldt, int64_t K, const int32_t *__restrict__ probe_id,
    const float *__restrict__ probe_d, int P, int L, const int32_t *__restrict__ nbr,
    const float *__restrict__ cst, const float *__restrict__ alpha, int S,
    const uint4 *__restrict__ sub_info,
    SubDesc *__restrict__ desc, int64_t *__restrict__ kept_sub, int64_t *__restrict__ n_scanned,
    int64_t nq, const float *__restrict__ Qt, int D, int M, const float *__restrict__ codebook,
    float *__restrict__ lut)
{
    extern __shared__ __attribute__((aligned(16))) uint32_t dyn[];
    if ((int64_t)blockIdx.x >= nq) {   // (uniform) a table workgroup
        const int64_t ql = (int64_t)blockIdx.x - nq;
        lut_body<BLOCK>(Qt + ql * D, D, M, codebook, lut + ql * (int64_t)M * 256, reinterpret_cast<float *>(dyn));
        return;
    }
    score_prune_body<BLOCK, MAXV>(Dt, ldt, K, probe_id, probe_d, P, L, nbr, cst, alpha, S, sub_info, desc, kept_sub, n_scanned,
                                  blockIdx.x, dyn);
}

// Rotation in front of the product quantiser (Section 4: OPQ-compressed displacements, one global
// rotation): Y[i] = R X[i] for n rows of D floats, with Rt = R transposed ([b][a] = R[a][b]) so
// that consecutive lanes read consecutive words.  A workgroup takes ROT_ROWS rows into LDS and
// every thread owns output components a = tid, tid + 256, ...; each component is one chain of
// fused multiply-adds in the order b = 0 .. D-1.  X and Y may be the same array (a workgroup reads
// its rows before it writes them).  Dynamic LDS: ROT_ROWS * D floats.
constexpr int ROT_ROWS = 16;

__global__ __launch_bounds__(256) void rotate_rows_kernel(const float *__restrict__ X, int64_t n, int D,
                                                          const float *__restrict__ Rt, float *__restrict__ Y)
{
    extern __shared__ float xs[];                       // [ROT_ROWS][D]
    const int64_t r0 = (int64_t)blockIdx.x * ROT_ROWS;
    const int rows = n - r0 < ROT_ROWS ? (int)(n - r0) : ROT_ROWS;
    for (int i = threadIdx.x; i < rows * D; i += 256) xs[i] = X[r0 * D + i];
    __syncthreads();
    for (int a = threadIdx.x; a < D; a += 256) {
        float acc[ROT_ROWS];
#pragma unroll
        for (int r = 0; r < ROT_ROWS; ++r) acc[r] = 0.f;
        for (int b = 0; b < D; ++b) {
            const float w = Rt[(int64_t)b * D + a];
#pragma unroll
            for (int r = 0; r < ROT_ROWS; ++r) acc[r] = fmaf(w, xs[r * D + b], acc[r]);   // rows past `rows` hold stale data, never stored
        }
        for (int r = 0; r < rows; ++r) Y[(r0 + r) * D + a] = acc[r];
    }
}

// out[b][a] = in[a][b] for a D x D matrix
__global__ __launch_bounds__(256) void transpose_square_kernel(const float *__restrict__ in, int D, float *__restrict__ out)
{
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i >= D * D) return;
    const int a = i / D, b = i - a * D;
    out[b * D + a] = in[i];
}

}  // namespace ivf
