// Index-time training kernels (Section 3.2 "The model" and "Learning the scaling factor",
// Section 2 for the PQ codebooks): a stable least-significant-digit radix sort that puts items into
// bucket order (the grouped layout, and the member lists of k-means clusters), segment sums in a
// fixed order (cluster means, the two sums of Eq. (12)), the neighbour table of Eq. (2), and the
// 256-level scalar quantiser.  Everything here is deterministic: no floating-point atomics, every
// sum is taken in an order that depends on the data layout only.
#pragma once
#include "util.hpp"

namespace ivf {

// ------------------------------------------------------------------ stable radix sort (8-bit digits)
constexpr int RS_BLOCK = 256;                 // threads per workgroup
constexpr int RS_ROUNDS = 16;                 // items per thread
constexpr int RS_TILE = RS_BLOCK * RS_ROUNDS; // consecutive items per workgroup

// Lanes of the wavefront whose digit equals this lane's (8 ballots).
__device__ __forceinline__ uint64_t match_digit(uint32_t digit, bool valid)
{
    uint64_t peers = __ballot(valid);
#pragma unroll
    for (int b = 0; b < 8; ++b) {
        const uint64_t m = __ballot((digit >> b) & 1u);
        peers &= ((digit >> b) & 1u) ? m : ~m;
    }
    return peers;
}

// hist[d * nblocks + block] = number of items of the workgroup's tile whose digit is d.
__global__ __launch_bounds__(RS_BLOCK) void radix_hist_kernel(const uint32_t *__restrict__ keys, int64_t n,
                                                              int shift, uint32_t *__restrict__ hist,
                                                              int64_t nblocks)
{
    __shared__ uint32_t h[256];
    const int tid = threadIdx.x;
    h[tid] = 0;
    __syncthreads();
    const int64_t base = (int64_t)blockIdx.x * RS_TILE;
#pragma unroll 4
    for (int r = 0; r < RS_ROUNDS; ++r) {
        const int64_t i = base + r * RS_BLOCK + tid;
        const bool valid = i < n;
        const uint32_t d = valid ? (keys[i] >> shift) & 255u : 0u;
        const uint64_t peers = match_digit(d, valid);
        if (valid && (peers & ((1ull << (tid & 63)) - 1ull)) == 0) atomicAdd(&h[d], (uint32_t)__popcll(peers));
    }
    __syncthreads();
    hist[(int64_t)tid * nblocks + blockIdx.x] = h[tid];
}

// Moves every item of the tile to base[d * nblocks + block] + (its rank among the tile's items with
// the same digit, in input order): a stable partition by the digit.  vals_in == NULL: the value of
// item i is i.
__global__ __launch_bounds__(RS_BLOCK) void radix_scatter_kernel(
    const uint32_t *__restrict__ keys_in, const uint32_t *__restrict__ vals_in, int64_t n, int shift,
    const uint32_t *__restrict__ base, int64_t nblocks, uint32_t *__restrict__ keys_out,
    uint32_t *__restrict__ vals_out)
{
    constexpr int NW = RS_BLOCK / WAVE;
    __shared__ uint32_t run[256];             // items of each digit placed by earlier rounds, plus the tile's base
    __shared__ uint32_t wcnt[NW][256];        // this round's items per wavefront and digit
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    run[tid] = base[(int64_t)tid * nblocks + blockIdx.x];
#pragma unroll
    for (int w = 0; w < NW; ++w) wcnt[w][tid] = 0;
    __syncthreads();
    const int64_t t0 = (int64_t)blockIdx.x * RS_TILE;
    for (int r = 0; r < RS_ROUNDS; ++r) {
        const int64_t i = t0 + r * RS_BLOCK + tid;
        const bool valid = i < n;
        const uint32_t key = valid ? keys_in[i] : 0u;
        const uint32_t val = valid ? (vals_in ? vals_in[i] : (uint32_t)i) : 0u;
        const uint32_t d = (key >> shift) & 255u;
        const uint64_t peers = match_digit(d, valid);
        const uint32_t rank = (uint32_t)__popcll(peers & ((1ull << lane) - 1ull));
        if (valid && rank == 0) wcnt[wave][d] = (uint32_t)__popcll(peers);
        __syncthreads();
        if (valid) {
            uint32_t at = run[d] + rank;
#pragma unroll
            for (int w = 0; w < NW; ++w)
                if (w < wave) at += wcnt[w][d];
            keys_out[at] = key;
            if (vals_out) vals_out[at] = val;
        }
        __syncthreads();
        {
            uint32_t s = 0;
#pragma unroll
            for (int w = 0; w < NW; ++w) { s += wcnt[w][tid]; wcnt[w][tid] = 0; }
            run[tid] += s;
        }
        __syncthreads();
    }
}

// offsets[b] = first sorted position whose key is >= b, for b in [0, nbuckets]; keys ascending.
// Thread i covers the buckets in (key[i-1], key[i]]; the thread after the last item the rest.
__global__ __launch_bounds__(256) void bucket_offsets_kernel(const uint32_t *__restrict__ sorted_keys, int64_t n,
                                                             int64_t nbuckets, uint32_t *__restrict__ offsets)
{
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i > n) return;
    const int64_t lo = i == 0 ? 0 : (int64_t)sorted_keys[i - 1] + 1;
    const int64_t hi = i == n ? nbuckets : (int64_t)sorted_keys[i];
    for (int64_t b = lo; b <= hi && b <= nbuckets; ++b) offsets[b] = (uint32_t)i;
}

__global__ __launch_bounds__(256) void fill_u64_kernel(unsigned long long *__restrict__ v, int64_t n, unsigned long long x)
{
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i < n) v[i] = x;
}

__global__ __launch_bounds__(256) void iota_u32_kernel(uint32_t *__restrict__ v, int64_t n)
{
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i < n) v[i] = (uint32_t)i;
}

// bucket[i] = region[i] * L + sub[i]: the subregion a point is stored in (Section 3.2, grouped storage)
__global__ __launch_bounds__(256) void bucket_ids_kernel(const int32_t *__restrict__ region, const int32_t *__restrict__ sub,
                                                         int64_t n, int L, int32_t *__restrict__ bucket)
{
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i < n) bucket[i] = region[i] * L + sub[i];
}

// keys[i] = byte m of row i of an [n][M] byte matrix
__global__ __launch_bounds__(256) void byte_column_kernel(const uint8_t *__restrict__ codes, int64_t n, int M, int m,
                                                          uint32_t *__restrict__ keys)
{
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i < n) keys[i] = codes[i * M + m];
}

// order-preserving keys of floats, and back
__global__ __launch_bounds__(256) void float_keys_kernel(const float *__restrict__ v, int64_t n, uint32_t *__restrict__ keys)
{
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i < n) keys[i] = float_key(v[i]);
}

__global__ __launch_bounds__(256) void key_floats_kernel(const uint32_t *__restrict__ keys, int64_t n, float *__restrict__ v)
{
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i < n) v[i] = key_float(keys[i]);
}

// dst row j = src row perm[j], rows of row_bytes bytes (16-byte pieces when everything is aligned)
__global__ __launch_bounds__(256) void gather_rows_kernel(const uint8_t *__restrict__ src, int64_t row_bytes,
                                                          const int32_t *__restrict__ perm, int64_t n,
                                                          uint8_t *__restrict__ dst, int vec)
{
    const int64_t per_row = row_bytes / vec;
    const int64_t t = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (t >= n * per_row) return;
    const int64_t j = t / per_row, c = t - j * per_row;
    const int64_t s = (int64_t)perm[j] * row_bytes + c * vec, d = j * row_bytes + c * vec;
    if (vec == 16) *reinterpret_cast<uint4 *>(dst + d) = *reinterpret_cast<const uint4 *>(src + s);
    else if (vec == 8) *reinterpret_cast<uint2 *>(dst + d) = *reinterpret_cast<const uint2 *>(src + s);
    else if (vec == 4) *reinterpret_cast<uint32_t *>(dst + d) = *reinterpret_cast<const uint32_t *>(src + s);
    else dst[d] = src[s];
}

// ------------------------------------------------------------------ segment sums in a fixed order
// Segment g holds the rows perm[off[g]] .. perm[off[g+1] - 1] (perm == NULL: the positions
// themselves) of X (row stride ld, columns col0 .. col0 + ncols - 1).  One workgroup per segment:
// thread t adds rows t, t + 256, ... of the segment in fp64, eight columns at a time, and the 256
// partial sums are combined by a tree whose shape does not depend on anything but the thread
// index, so the result is a function of the member list alone.
//   MODE 0: sum[g][c] (fp64) and cnt[g]
//   MODE 1: mean[g * ld_out + col0_out + c] = (float)(sum / count) for non-empty segments, empty ones are left alone
template <class T, int MODE>
__global__ __launch_bounds__(256) void segment_sum_kernel(const T *__restrict__ X, int64_t ld, int col0, int ncols,
                                                          const uint32_t *__restrict__ perm,
                                                          const uint32_t *__restrict__ off,
                                                          double *__restrict__ sum, float *__restrict__ mean,
                                                          int64_t ld_out, int col0_out)
{
    __shared__ double red[256][8];
    const int tid = threadIdx.x;
    const int64_t g = blockIdx.x;
    const uint32_t b = off[g], e = off[g + 1];
    for (int c0 = 0; c0 < ncols; c0 += 8) {
        double acc[8] = {0, 0, 0, 0, 0, 0, 0, 0};
        for (uint32_t j = b + tid; j < e; j += 256) {
            const int64_t row = perm ? (int64_t)perm[j] : (int64_t)j;
            const T *p = X + row * ld + col0 + c0;
#pragma unroll
            for (int c = 0; c < 8; ++c)
                if (c0 + c < ncols) acc[c] += (double)p[c];
        }
#pragma unroll
        for (int c = 0; c < 8; ++c) red[tid][c] = acc[c];
        __syncthreads();
        for (int s = 128; s > 0; s >>= 1) {
            if (tid < s)
#pragma unroll
                for (int c = 0; c < 8; ++c) red[tid][c] += red[tid + s][c];
            __syncthreads();
        }
        if (tid < 8 && c0 + tid < ncols) {
            if (MODE == 0) sum[g * ncols + c0 + tid] = red[0][tid];
            else if (e > b) mean[g * ld_out + col0_out + c0 + tid] = (float)(red[0][tid] / (double)(e - b));
        }
        __syncthreads();
    }
}

// out[0] = sum of v[0..n) in fp64 by one workgroup, fixed order (thread t adds t, t + 1024, ...; tree).
template <class T>
__global__ __launch_bounds__(1024) void fixed_sum_kernel(const T *__restrict__ v, int64_t n, double *__restrict__ out)
{
    __shared__ double red[1024];
    const int tid = threadIdx.x;
    double a = 0.0;
    for (int64_t i = tid; i < n; i += 1024) a += (double)v[i];
    red[tid] = a;
    __syncthreads();
    for (int s = 512; s > 0; s >>= 1) {
        if (tid < s) red[tid] += red[tid + s];
        __syncthreads();
    }
    if (tid == 0) out[0] = red[0];
}

// out[b] = sum over i < n of v[i * stride + b], b = blockIdx.x < stride, fixed order
__global__ __launch_bounds__(1024) void strided_sum_kernel(const double *__restrict__ v, int64_t n, int stride,
                                                          double *__restrict__ out)
{
    __shared__ double red[1024];
    const int tid = threadIdx.x, b = blockIdx.x;
    double a = 0.0;
    for (int64_t i = tid; i < n; i += 1024) a += v[i * stride + b];
    red[tid] = a;
    __syncthreads();
    for (int s = 512; s > 0; s >>= 1) {
        if (tid < s) red[tid] += red[tid + s];
        __syncthreads();
    }
    if (tid == 0) out[b] = red[0];
}

// rows init_idx[j] of X [.][ld] (columns col0 .. col0+ncols) -> out[j][ncols]
__global__ __launch_bounds__(256) void take_rows_kernel(const float *__restrict__ X, int64_t ld, int col0, int ncols,
                                                        const int64_t *__restrict__ idx, int64_t k,
                                                        float *__restrict__ out, int64_t ld_out, int col0_out)
{
    const int64_t t = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (t >= k * ncols) return;
    const int64_t j = t / ncols, c = t - j * ncols;
    out[j * ld_out + col0_out + c] = X[idx[j] * ld + col0 + c];
}

// ------------------------------------------------------------------ alpha (Eqs. (10)-(12))
// Step 1 per training point (one wavefront each): the neighbour whose line through c leaves the
// smallest residual with the coefficient clamped to [0, 1] (lowest l on ties); stat[i] = {(x-c)^T(s-c), ||s-c||^2}.
__global__ __launch_bounds__(64) void alpha_point_kernel(
    const float *__restrict__ X, int64_t n, int D, int L, const int32_t *__restrict__ region,
    const float *__restrict__ C, const int32_t *__restrict__ nbr, double *__restrict__ stat)
{
    extern __shared__ float sm[];
    float *xc = sm;   // x - c
    const int lane = threadIdx.x;
    const int64_t i = blockIdx.x;
    if (i >= n) return;
    const int64_t r = region[i];
    for (int t = lane; t < D; t += WAVE) xc[t] = X[i * D + t] - C[r * D + t];
    wave_sync();
    double xc2 = 0.0;
    for (int t = 0; t < D; ++t) xc2 += (double)xc[t] * (double)xc[t];
    double best = INFINITY, bdot = 0.0, bn2 = 0.0;
    int bl = 0x7fffffff;
    for (int l = lane; l < L; l += WAVE) {
        const float *s = C + (int64_t)nbr[r * L + l] * D;
        const float *c = C + r * D;
        double dot = 0.0, n2 = 0.0;
        for (int t = 0; t < D; ++t) {
            double u = (double)s[t] - (double)c[t];
            dot += (double)xc[t] * u;
            n2 += u * u;
        }
        double a = n2 > 0.0 ? dot / n2 : 0.0;
        a = a < 0.0 ? 0.0 : (a > 1.0 ? 1.0 : a);
        double res = xc2 - 2.0 * a * dot + a * a * n2;
        if (res < best) { best = res; bl = l; bdot = dot; bn2 = n2; }
    }
    double wbest = best;
    int wl = bl;
    wave_argmin(wbest, wl);
    if (bl == wl && wl != 0x7fffffff) {   // the single lane holding the winner
        stat[2 * i] = bdot;
        stat[2 * i + 1] = bn2;
    }
}

// Step 2: alpha_r = clamp(num_r / den_r) from the per-region sums nd[r] = {num, den}; regions without
// training points or with a zero denominator get the pooled ratio tot[0] / tot[1].
__global__ __launch_bounds__(256) void alpha_finish_kernel(const double *__restrict__ nd, const double *__restrict__ tot,
                                                           int64_t K, float *__restrict__ alpha)
{
    const int64_t r = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (r >= K) return;
    double pooled = tot[1] > 0.0 ? tot[0] / tot[1] : 0.0;
    pooled = pooled < 0.0 ? 0.0 : (pooled > 1.0 ? 1.0 : pooled);
    double a = nd[2 * r + 1] > 0.0 ? nd[2 * r] / nd[2 * r + 1] : pooled;
    a = a < 0.0 ? 0.0 : (a > 1.0 ? 1.0 : a);
    alpha[r] = (float)a;
}

// ------------------------------------------------------------------ neighbour table (Eq. (2))
// Row r of the P = L + 1 nearest centroids of centroid r (ascending id, with distances) -> its L
// neighbours ordered by (distance, id) without r itself; if r is not in its own list (more than L
// exact duplicates of it come first) the entry that is last in (distance, id) order is dropped.
// One wavefront per row; rank of an entry = number of entries with a smaller (distance, id) key.
__global__ __launch_bounds__(64) void neighbour_rows_kernel(const int32_t *__restrict__ top_id,
                                                            const float *__restrict__ top_d, int64_t K, int P,
                                                            int32_t *__restrict__ nbr, float *__restrict__ cs)
{
    extern __shared__ unsigned long long nk[];   // P keys
    const int lane = threadIdx.x;
    const int64_t r = blockIdx.x;
    if (r >= K) return;
    const int L = P - 1;
    bool has_self = false;
    for (int j = lane; j < P; j += WAVE) {
        const int32_t id = top_id[r * P + j];
        unsigned long long key = ((unsigned long long)float_key(top_d[r * P + j]) << 32) | (uint32_t)id;
        if (id == (int32_t)r) { key = ~0ull; has_self = true; }
        nk[j] = key;
    }
    has_self = __ballot(has_self) != 0;
    wave_sync();
    for (int j = lane; j < P; j += WAVE) {
        const unsigned long long key = nk[j];
        if (key == ~0ull) continue;                  // the centroid itself
        int rank = 0;
        for (int t = 0; t < P; ++t) rank += nk[t] < key ? 1 : 0;
        if (rank < L) {                              // without self in the list the largest key has rank L: dropped
            nbr[r * L + rank] = (int32_t)(uint32_t)key;
            cs[r * L + rank] = key_float((uint32_t)(key >> 32));
        }
    }
    (void)has_self;
}

// ------------------------------------------------------------------ scalar quantiser (256 levels)
// label[i] = nearest entry of the ascending table to s[i] in fp64, lowest index on ties
__global__ __launch_bounds__(256) void lloyd1d_label_kernel(const float *__restrict__ s, int64_t n,
                                                            const float *__restrict__ table, uint32_t *__restrict__ label)
{
    __shared__ double tab[256];
    tab[threadIdx.x] = (double)table[threadIdx.x];
    __syncthreads();
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (int64_t)gridDim.x * 256) {
        const double v = (double)s[i];
        double best = INFINITY;
        int bj = 0;
        for (int j = 0; j < 256; ++j) {
            const double d = fabs(v - tab[j]);
            if (d < best) { best = d; bj = j; }
        }
        label[i] = (uint32_t)bj;
    }
}

// table[j] = s[floor((j + 1/2) / 256 * n)] of the ascending s
__global__ __launch_bounds__(256) void lloyd1d_init_kernel(const float *__restrict__ s, int64_t n, float *__restrict__ table)
{
    const int j = threadIdx.x;
    int64_t p = (int64_t)(((double)j + 0.5) / 256.0 * (double)n);
    if (p >= n) p = n - 1;
    table[j] = s[p];
}

// new levels: the mean of each level's values (sum[j] over off[j+1] - off[j] values), a level without
// values keeps its entry; sorted ascending (bitonic, one workgroup of 256), rounded to fp32.
__global__ __launch_bounds__(256) void lloyd1d_update_kernel(const double *__restrict__ sum, const uint32_t *__restrict__ off,
                                                             float *__restrict__ table)
{
    __shared__ double lev[256];
    const int j = threadIdx.x;
    const uint32_t cnt = off[j + 1] - off[j];
    lev[j] = cnt > 0 ? sum[j] / (double)cnt : (double)table[j];
    for (int size = 2; size <= 256; size <<= 1)
        for (int stride = size >> 1; stride > 0; stride >>= 1) {
            __syncthreads();
            if (j < 128) {
                const int a = 2 * j - (j & (stride - 1)), b = a + stride;
                const bool up = (a & size) == 0;
                const double x = lev[a], y = lev[b];
                if ((x > y) == up) { lev[a] = y; lev[b] = x; }
            }
        }
    __syncthreads();
    table[j] = (float)lev[j];
}

}  // namespace ivf
