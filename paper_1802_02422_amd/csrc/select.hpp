// Exact selection of the nsel smallest of n items by (key, position) inside
// one workgroup: an MSB-first radix select on order-preserving uint32 keys
// followed by an ordered compaction, so the winners come out in ascending
// position and ties on the key resolve to the lowest positions.
#pragma once
#include "util.hpp"

namespace ivf {

struct SelectShared {
    uint32_t hist[4][256];   // one histogram per radix pass
    uint32_t scan[16];
    uint32_t pick[4][2];
};

// hist[bin] += 1 for the calling lanes.  Keys that share their leading bytes (distances of one
// query) put whole wavefronts into one bin of the first passes; 64 atomics on one LDS word are
// executed one after the other, so a wavefront whose lanes all agree adds its population count once.
__device__ __forceinline__ void hist_add(uint32_t *hist, uint32_t bin)
{
    const uint32_t b0 = (uint32_t)__builtin_amdgcn_readfirstlane((int)bin);
    const uint64_t active = __ballot(true), same = __ballot(bin == b0);
    if (same == active) {
        if (__builtin_amdgcn_mbcnt_hi((uint32_t)(active >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)active, 0u)) == 0)
            atomicAdd(&hist[b0], (uint32_t)__popcll(active));
    } else {
        atomicAdd(&hist[bin], 1u);
    }
}

// Finds the key value `pivot` of the nsel-th smallest item and the number
// `need` of items equal to pivot that belong to the selection (those at the
// lowest positions).  key(i) must be pure.  1 <= nsel <= n.
template <int BLOCK, class KeyFn>
__device__ void block_radix_select(KeyFn key, int64_t n, uint32_t nsel, SelectShared &sh,
                                   uint32_t &pivot, uint32_t &need)
{
    const int tid = threadIdx.x;
    uint32_t prefix = 0, mask = 0, remaining = nsel;
    __syncthreads();                              // the previous user of sh is done
    for (int i = tid; i < 4 * 256; i += BLOCK) (&sh.hist[0][0])[i] = 0;
    __syncthreads();
    for (int pass = 0; pass < 4; ++pass) {        // two barriers per pass
        const int shift = 24 - 8 * pass;
        uint32_t *hist = sh.hist[pass];
        // several independent key reads in flight per thread before their histogram updates
        int64_t i = tid;
        for (; i + 3 * BLOCK < n; i += 4 * BLOCK) {
            uint32_t k[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) k[u] = key(i + u * BLOCK);
#pragma unroll
            for (int u = 0; u < 4; ++u)
                if ((k[u] & mask) == prefix) hist_add(hist, (k[u] >> shift) & 255u);
        }
        for (; i < n; i += BLOCK) {
            uint32_t k = key(i);
            if ((k & mask) == prefix) hist_add(hist, (k >> shift) & 255u);
        }
        __syncthreads();
        if (tid < WAVE) {
            uint32_t c[4], s = 0;
#pragma unroll
            for (int j = 0; j < 4; ++j) { c[j] = hist[4 * tid + j]; s += c[j]; }
            uint32_t inc = wave_inclusive_scan(s);
            uint32_t exc = inc - s;
            if (exc < remaining && inc >= remaining) {   // exactly one lane
                uint32_t cum = exc;
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    if (cum < remaining && cum + c[j] >= remaining) {
                        sh.pick[pass][0] = 4 * tid + j;
                        sh.pick[pass][1] = remaining - cum;
                    }
                    cum += c[j];
                }
            }
        }
        __syncthreads();
        prefix |= sh.pick[pass][0] << shift;
        mask |= 0xFFu << shift;
        remaining = sh.pick[pass][1];
    }
    pivot = prefix;
    need = remaining;
}

// Calls emit(out_pos, i, key) for every item with key < pivot and for the
// `need` lowest-positioned items with key == pivot, where out_pos is the item's
// rank among the emitted ones in ascending i.  Stops early once nsel items
// have been emitted.  Returns the number emitted.
template <int BLOCK, class KeyFn, class EmitFn>
__device__ uint32_t block_emit_selected(KeyFn key, int64_t n, uint32_t nsel, uint32_t pivot,
                                        uint32_t need, SelectShared &sh, EmitFn emit)
{
    const int tid = threadIdx.x;
    uint32_t run_lt = 0, run_eq = 0;
    for (int64_t base = 0; base < n; base += BLOCK) {
        int64_t i = base + tid;
        bool valid = i < n;
        uint32_t k = valid ? key(i) : 0u;
        bool lt = valid && k < pivot, eq = valid && k == pivot;
        uint32_t packed = (lt ? 1u : 0u) | (eq ? 0x10000u : 0u), total;
        uint32_t exc = block_exclusive_scan<BLOCK>(packed, sh.scan, total);
        uint32_t lt_ex = exc & 0xFFFFu, eq_ex = run_eq + (exc >> 16);
        if (lt) {
            emit(run_lt + lt_ex + (eq_ex < need ? eq_ex : need), i, k);
        } else if (eq && eq_ex < need) {
            emit(run_lt + lt_ex + eq_ex, i, k);
        }
        run_lt += total & 0xFFFFu;
        run_eq += total >> 16;
        if (run_lt + (run_eq < need ? run_eq : need) >= nsel) break;   // uniform
    }
    return run_lt + (run_eq < need ? run_eq : need);
}

// The same selection for keys held in LDS (16-byte aligned, readable up to the next multiple of
// four past n): every thread owns a contiguous run of items, reads it once with 128-bit loads
// into registers (a run per thread read word by word would put 16 lanes on every bank), counts
// its selected items, one workgroup scan turns the counts into output offsets, and the thread
// emits its run in order.  One scan instead of one per BLOCK items.  n <= 4 * MAXV * BLOCK (MAXV:
// 128-bit words per thread), n < 65536.  Every key has been read into registers when the first
// emit runs: emit may overwrite the array.
template <int BLOCK, int MAXV = 8, class EmitFn>
__device__ uint32_t block_emit_selected_runs(const uint32_t *keys, int n, uint32_t pivot, uint32_t need,
                                             SelectShared &sh, EmitFn emit)
{
    const int ipt = ((n + BLOCK - 1) / BLOCK + 3) & ~3;       // items per thread, a multiple of 4
    const int i0 = threadIdx.x * ipt;
    uint32_t kv[4 * MAXV];
    uint32_t lt = 0, eq = 0;
#pragma unroll
    for (int v = 0; v < MAXV; ++v) {
        uint4 w = make_uint4(0xFFFFFFFFu, 0xFFFFFFFFu, 0xFFFFFFFFu, 0xFFFFFFFFu);
        if (4 * v < ipt && i0 + 4 * v < n) w = *reinterpret_cast<const uint4 *>(&keys[i0 + 4 * v]);
        kv[4 * v + 0] = w.x; kv[4 * v + 1] = w.y; kv[4 * v + 2] = w.z; kv[4 * v + 3] = w.w;
    }
    bool in[4 * MAXV];
#pragma unroll
    for (int j = 0; j < 4 * MAXV; ++j) {
        in[j] = j < ipt && i0 + j < n;
        lt += (in[j] && kv[j] < pivot) ? 1u : 0u;
        eq += (in[j] && kv[j] == pivot) ? 1u : 0u;
    }
    uint32_t total;
    const uint32_t exc = block_exclusive_scan<BLOCK>(lt | (eq << 16), sh.scan, total);
    uint32_t lt_seen = exc & 0xFFFFu, eq_seen = exc >> 16;
#pragma unroll
    for (int j = 0; j < 4 * MAXV; ++j) {
        if (!in[j]) continue;
        const uint32_t k = kv[j];
        if (k < pivot) {
            emit(lt_seen + (eq_seen < need ? eq_seen : need), (int64_t)(i0 + j), k);
            ++lt_seen;
        } else if (k == pivot) {
            if (eq_seen < need) emit(lt_seen + eq_seen, (int64_t)(i0 + j), k);
            ++eq_seen;
        }
    }
    const uint32_t tl = total & 0xFFFFu, te = total >> 16;
    return tl + (te < need ? te : need);
}

// In-place ascending bitonic sort of n (a power of two) uint64 keys in LDS by
// the whole workgroup.
template <int BLOCK>
__device__ void block_bitonic_sort(uint64_t *a, int n)
{
    for (int size = 2; size <= n; size <<= 1)
        for (int stride = size >> 1; stride > 0; stride >>= 1) {
            __syncthreads();
            for (int t = threadIdx.x; t < n / 2; t += BLOCK) {
                int i = 2 * t - (t & (stride - 1)), j = i + stride;
                bool up = (i & size) == 0;
                uint64_t x = a[i], y = a[j];
                if ((x > y) == up) { a[i] = y; a[j] = x; }
            }
        }
    __syncthreads();
}

// The same for one wavefront on its private LDS array.
__device__ __forceinline__ void wave_bitonic_sort(uint64_t *a, int n)
{
    const int lane = threadIdx.x & (WAVE - 1);
    for (int size = 2; size <= n; size <<= 1)
        for (int stride = size >> 1; stride > 0; stride >>= 1) {
            wave_sync();
            for (int t = lane; t < n / 2; t += WAVE) {
                int i = 2 * t - (t & (stride - 1)), j = i + stride;
                bool up = (i & size) == 0;
                uint64_t x = a[i], y = a[j];
                if ((x > y) == up) { a[i] = y; a[j] = x; }
            }
        }
    wave_sync();
}

}  // namespace ivf
