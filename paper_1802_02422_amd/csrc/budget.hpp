// Candidate budget (Section 4 evaluates candidate lists of a given length R): of the subregions
// that survived the pruning, only a prefix in ascending order of (Eq. (7) distance, subregion id)
// is scanned, up to and including the subregion with which the points collected reach R.
#pragma once
#include "query.hpp"

namespace ivf {

// One workgroup per query, after score_prune_kernel has written the query's S descriptors (in
// ascending subregion id).  A subregion is visited iff the subregions before it in (score,
// id) order hold fewer than R points together.  The score of the crossing subregion is found by an
// MSB-first radix search on the order-preserving score keys in which a histogram bin weighs the
// points of its subregions; among subregions that tie with it the order is position order (= id
// order), resolved by one ordered scan.  The length of every subregion that is not visited is
// set to 0 (the scan skips empty descriptors), visited[q][i] (may be NULL) receives the flags and
// n_scanned[q] (may be NULL) the number of points of the visited subregions.
template <int BLOCK>
__global__ __launch_bounds__(BLOCK) void budget_cut_kernel(SubDesc *__restrict__ desc, int S, uint32_t R,
                                                           uint8_t *__restrict__ visited,
                                                           int64_t *__restrict__ n_scanned)
{
    __shared__ uint32_t hist[256];
    __shared__ uint32_t scan_s[BLOCK / WAVE];
    __shared__ uint32_t pick[2];
    __shared__ unsigned long long total_s;
    const int tid = threadIdx.x;
    const int64_t q = blockIdx.x;
    SubDesc *d = desc + q * S;
    uint32_t prefix = 0, mask = 0, remaining = R;
    bool all = false;
    if (tid == 0) total_s = 0;
    for (int pass = 0; pass < 4; ++pass) {
        const int shift = 24 - 8 * pass;
        for (int i = tid; i < 256; i += BLOCK) hist[i] = 0;
        __syncthreads();
        for (int i = tid; i < S; i += BLOCK) {
            const uint32_t k = float_key(d[i].base), len = d[i].len;
            if (len && (k & mask) == prefix) atomicAdd(&hist[(k >> shift) & 255u], len);
        }
        __syncthreads();
        if (tid < WAVE) {
            uint32_t c[4], s = 0;
#pragma unroll
            for (int j = 0; j < 4; ++j) { c[j] = hist[4 * tid + j]; s += c[j]; }
            const uint32_t inc = wave_inclusive_scan(s);
            const uint32_t exc = inc - s;
            const uint32_t tot = (uint32_t)__builtin_amdgcn_readlane((int)inc, WAVE - 1);
            if (tot < remaining) {                       // (first pass only) fewer than R points in all: visit everything
                if (tid == 0) { pick[0] = 256u; pick[1] = 0u; }
            } else if (exc < remaining && inc >= remaining) {   // exactly one lane
                uint32_t cum = exc;
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    if (cum < remaining && cum + c[j] >= remaining) {
                        pick[0] = 4 * tid + j;
                        pick[1] = remaining - cum;
                    }
                    cum += c[j];
                }
            }
        }
        __syncthreads();
        if (pick[0] == 256u) { all = true; break; }      // uniform
        prefix |= pick[0] << shift;
        mask |= 0xFFu << shift;
        remaining = pick[1];
        __syncthreads();                                 // pick is rewritten by the next pass
    }
    // prefix: score key of the crossing subregion; remaining (> 0): points still wanted from the subregions with that key
    uint32_t run = 0;
    unsigned long long mine = 0;
    for (int base = 0; base < S; base += BLOCK) {
        const int i = base + tid;
        const bool valid = i < S;
        const uint32_t k = valid ? float_key(d[i].base) : 0xFFFFFFFFu;
        const uint32_t len = valid ? d[i].len : 0u;
        const bool eq = valid && !all && k == prefix;
        uint32_t tot;
        const uint32_t before = run + block_exclusive_scan<BLOCK>(eq ? len : 0u, scan_s, tot);
        run += tot;
        if (valid) {
            const bool vis = all || k < prefix || (eq && before < remaining);
            if (!vis) d[i].len = 0u;
            else mine += len;
            if (visited) visited[q * S + i] = vis ? 1 : 0;
        }
    }
    if (n_scanned) {
        if (mine) atomicAdd(&total_s, mine);
        __syncthreads();
        if (tid == 0) n_scanned[q] = (int64_t)total_s;
    }
}

}  // namespace ivf
