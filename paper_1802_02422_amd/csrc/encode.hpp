// Index-time kernels: subregion assignment (Eq. (3)), displacement (Eq. (4)),
// PQ encoding, the per-point constant of Eq. (6), and the statistics for
// learning alpha (Eqs. (11)-(12)).  One wavefront per point.
#pragma once
#include "util.hpp"

namespace ivf {

// LDS per workgroup (one wavefront): x, c and e/mu, each D floats.  With codebook == NULL the
// kernel stops after the displacement (written to out_res, the subcentroid to out_mu).
__global__ __launch_bounds__(64) void encode_kernel(
    const float *__restrict__ X, int64_t n, int D, int M, int L, const int32_t *__restrict__ region,
    const float *__restrict__ C, const int32_t *__restrict__ nbr, const float *__restrict__ alpha,
    const float *__restrict__ cs_dist2, const float *__restrict__ codebook,
    const float *__restrict__ const_table, int32_t *__restrict__ out_sub,
    uint8_t *__restrict__ out_codes, uint8_t *__restrict__ out_byte, float *__restrict__ out_t,
    float *__restrict__ out_res, float *__restrict__ out_mu)
{
    extern __shared__ __attribute__((aligned(16))) float sm[];
    float *xs = sm, *cs = sm + D, *es = sm + 2 * D, *mus = sm + 3 * D;   // D is a multiple of 4: all 16-byte aligned
    const int lane = threadIdx.x;
    const int64_t i = blockIdx.x;
    if (i >= n) return;
    const int64_t r = region[i];
    const float a = alpha[r];
    for (int t = lane; t < D; t += WAVE) {
        xs[t] = X[i * D + t];
        cs[t] = C[r * D + t];
    }
    wave_sync();

    // Eq. (3) through the closed form of the subcentroid distance:
    // ||x - mu_l||^2 = (1-a)||x-c||^2 + a||x-s_l||^2 - a(1-a)||c-s_l||^2
    // Four neighbour rows at a time, 16 lanes per row, a lane taking every 16th group of four
    // components: a load instruction then reads four rows of up to 256 contiguous bytes (with a
    // lane per neighbour it touched 64 different rows, and the kernel was bounded by the number
    // of cache lines its loads addressed).
    const int D4 = D >> 2;
    const int g = lane >> 4, c16 = lane & 15;
    float dxc = 0.f;
    for (int cc = lane; cc < D4; cc += WAVE) {
        const float4 xv = *reinterpret_cast<const float4 *>(xs + 4 * cc);
        const float4 cv = *reinterpret_cast<const float4 *>(cs + 4 * cc);
        const float u0 = xv.x - cv.x, u1 = xv.y - cv.y, u2 = xv.z - cv.z, u3 = xv.w - cv.w;
        dxc = fmaf(u0, u0, dxc);
        dxc = fmaf(u1, u1, dxc);
        dxc = fmaf(u2, u2, dxc);
        dxc = fmaf(u3, u3, dxc);
    }
    dxc = wave_sum(dxc);
    float best = INFINITY;
    int best_l = 0x7fffffff;
    for (int lb = 0; lb < L; lb += WAVE) {            // 64 neighbours at a time: their ids in one load
        const int my_nbr = lb + lane < L ? nbr[r * L + lb + lane] : 0;
        const float my_cs = lb + lane < L ? cs_dist2[r * L + lb + lane] : 0.f;
        const int nl = L - lb < WAVE ? L - lb : WAVE;
        for (int l0 = 0; l0 < nl; l0 += 16) {         // four steps of four rows, their loads issued together
            float4 sv[4][2];
            const float4 *s4[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int64_t row = __shfl(my_nbr, (l0 + 4 * u + g) & (WAVE - 1), WAVE);
                s4[u] = reinterpret_cast<const float4 *>(C + row * D);
                const bool live = l0 + 4 * u + g < nl;
                sv[u][0] = live && c16 < D4 ? s4[u][c16] : make_float4(0.f, 0.f, 0.f, 0.f);
                sv[u][1] = live && c16 + 16 < D4 ? s4[u][c16 + 16] : make_float4(0.f, 0.f, 0.f, 0.f);
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int lw = l0 + 4 * u + g;          // neighbour within this batch of 64
                const bool live = lw < nl;
                const float csl = __shfl(my_cs, lw & (WAVE - 1), WAVE);
                float dxs = 0.f;
                if (live) {
#pragma unroll
                    for (int h = 0; h < 2; ++h)
                        if (c16 + 16 * h < D4) {
                            const float4 xv = *reinterpret_cast<const float4 *>(xs + 4 * (c16 + 16 * h));
                            const float u0 = xv.x - sv[u][h].x, u1 = xv.y - sv[u][h].y, u2 = xv.z - sv[u][h].z,
                                        u3 = xv.w - sv[u][h].w;
                            dxs = fmaf(u0, u0, dxs);
                            dxs = fmaf(u1, u1, dxs);
                            dxs = fmaf(u2, u2, dxs);
                            dxs = fmaf(u3, u3, dxs);
                        }
                    for (int cc = c16 + 32; cc < D4; cc += 16) {   // D > 128
                        const float4 sw = s4[u][cc];
                        const float4 xv = *reinterpret_cast<const float4 *>(xs + 4 * cc);
                        const float u0 = xv.x - sw.x, u1 = xv.y - sw.y, u2 = xv.z - sw.z, u3 = xv.w - sw.w;
                        dxs = fmaf(u0, u0, dxs);
                        dxs = fmaf(u1, u1, dxs);
                        dxs = fmaf(u2, u2, dxs);
                        dxs = fmaf(u3, u3, dxs);
                    }
                }
#pragma unroll
                for (int o = 8; o > 0; o >>= 1) dxs += __shfl_xor(dxs, o, WAVE);   // over the 16 lanes of the row
                if (live && c16 == 0) {
                    const float sc = fmaf(a, dxs, fmaf(1.f - a, dxc, -a * (1.f - a) * csl));
                    if (sc < best) { best = sc; best_l = lb + lw; }
                }
            }
        }
    }
    wave_argmin(best, best_l);
    if (lane == 0) out_sub[i] = best_l;

    // Eq. (4): displacement from the chosen subcentroid
    const float *s = C + (int64_t)nbr[r * L + best_l] * D;
    for (int t = lane; t < D; t += WAVE) {
        float mu = fmaf(a, s[t] - cs[t], cs[t]);
        mus[t] = mu;
        es[t] = xs[t] - mu;
        if (out_res) out_res[i * D + t] = xs[t] - mu;
        if (out_mu) out_mu[i * D + t] = mu;
    }
    wave_sync();
    if (!codebook) return;   // trained up to alpha only, or the codes are left to pq_encode_kernel

    // PQ: nearest of the 256 codewords per block of D/M dims, lowest index on ties
    const int ds = D / M;
    float tpart = 0.f;   // lane-partial of 2<mu, r> + ||r||^2
    for (int m = 0; m < M; ++m) {
        float bd = INFINITY;
        int bj = 0x7fffffff;
        for (int j = lane; j < 256; j += WAVE) {
            const float *cw = codebook + ((int64_t)m * 256 + j) * ds;
            float dd = 0.f;
            for (int t = 0; t < ds; ++t) {
                float u = es[m * ds + t] - cw[t];
                dd = fmaf(u, u, dd);
            }
            if (dd < bd) { bd = dd; bj = j; }
        }
        wave_argmin(bd, bj);
        if (lane == 0) out_codes[i * M + m] = (uint8_t)bj;
        const float *cw = codebook + ((int64_t)m * 256 + bj) * ds;
        for (int t = lane; t < ds; t += WAVE) {
            float rv = cw[t];
            tpart = fmaf(2.f * mus[m * ds + t], rv, fmaf(rv, rv, tpart));
        }
    }
    float tval = wave_sum(tpart);
    if (lane == 0 && out_t) out_t[i] = tval;

    if (const_table) {
        float bd = INFINITY;
        int bj = 0x7fffffff;
        for (int j = lane; j < 256; j += WAVE) {
            float dd = fabsf(tval - const_table[j]);
            if (dd < bd) { bd = dd; bj = j; }
        }
        wave_argmin(bd, bj);
        if (lane == 0) out_byte[i] = (uint8_t)bj;
    }
}

// PQ encoding of displacements, one THREAD per point with the whole codebook in LDS (M * 256 * DS
// floats, DS = D / M): all lanes walk the 256 codewords of a block together, so every codeword
// is one broadcast LDS read, the running minimum stays in the lane (no cross-lane reduction), and
// the arithmetic per (point, codeword) is the same sequence of fused multiply-adds as in
// encode_kernel: the codes are identical.  Also the per-point constant t = 2<mu, r> + ||r||^2
// of Eq. (6) and its nearest table entry, lowest index on ties.  E and MU are [n][D] fp32 (MU == NULL: codes only, the assignment step of the codebook training).
// A workgroup encodes several batches of blockDim.x points (grid-stride).
template <int DS>
__global__ __launch_bounds__(1024) void pq_encode_kernel(
    const float *__restrict__ E, const float *__restrict__ MU, int64_t n, int M,
    const float *__restrict__ codebook, const float *__restrict__ const_table,
    uint8_t *__restrict__ out_codes, uint8_t *__restrict__ out_byte, float *__restrict__ out_t)
{
    extern __shared__ __attribute__((aligned(16))) float cb[];   // M * 256 * DS
    __shared__ float tab[256];
    const int D = M * DS;
    for (int i = threadIdx.x; i < M * 256 * DS; i += blockDim.x) cb[i] = codebook[i];
    if (threadIdx.x < 256) tab[threadIdx.x] = const_table ? const_table[threadIdx.x] : 0.f;
    __syncthreads();
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x) {
        float tval = 0.f;
        for (int m = 0; m < M; ++m) {
            float ev[DS];
#pragma unroll
            for (int t = 0; t < DS; ++t) ev[t] = E[i * D + m * DS + t];
            float bd = INFINITY;
            int bj = 0;
            const float *cwm = cb + m * 256 * DS;
#pragma unroll 4
            for (int j = 0; j < 256; ++j) {
                float dd = 0.f;
#pragma unroll
                for (int t = 0; t < DS; ++t) {
                    const float u = ev[t] - cwm[j * DS + t];
                    dd = fmaf(u, u, dd);
                }
                if (dd < bd) { bd = dd; bj = j; }   // ascending j: lowest index on ties
            }
            out_codes[i * M + m] = (uint8_t)bj;
            const float *cw = cwm + bj * DS;
            if (MU) {
#pragma unroll
                for (int t = 0; t < DS; ++t) {
                    const float rv = cw[t];
                    tval = fmaf(2.f * MU[i * D + m * DS + t], rv, fmaf(rv, rv, tval));
                }
            }
        }
        if (out_t) out_t[i] = tval;
        if (const_table) {
            float bd = INFINITY;
            int bj = 0;
            for (int j = 0; j < 256; ++j) {
                const float dd = fabsf(tval - tab[j]);
                if (dd < bd) { bd = dd; bj = j; }
            }
            out_byte[i] = (uint8_t)bj;
        }
    }
}

}  // namespace ivf
