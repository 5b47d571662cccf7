// Stages 5-6: the asymmetric-distance scan of the kept subregions with
// per-wavefront top-k pools (Eq. (6)), and the final k-select.
//
// Record layout (built at load time): subregion b owns a 16-byte aligned block
// at byte offset BLK_ALIGN*blk_off[b] holding len*M code bytes followed by len
// constant-term bytes, so one subregion is one contiguous HBM run.
#pragma once
#include "layout.hpp"
#include "query.hpp"

namespace ivf {

constexpr int SCAN_BLOCK = 256;
constexpr int SCAN_WAVES = SCAN_BLOCK / WAVE;

__host__ __device__ inline int pool_capacity(int k)
{
    int cap = 256;
    while (cap < 2 * k) cap <<= 1;
    return cap;
}

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
template <int M> struct CodeWord;
template <> struct CodeWord<16> { typedef u32x4 type; };
template <> struct CodeWord<8> { typedef u32x2 type; };

// 4 * (byte B of w) in one VALU instruction (SDWA byte select feeding a shift);
// `two` is a register holding 2.
template <int B>
__device__ __forceinline__ uint32_t byte_x4(uint32_t w, uint32_t two)
{
    uint32_t r;
    if (B == 0) asm("v_lshlrev_b32_sdwa %0, %1, %2 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:BYTE_0" : "=v"(r) : "v"(two), "v"(w));
    if (B == 1) asm("v_lshlrev_b32_sdwa %0, %1, %2 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:BYTE_1" : "=v"(r) : "v"(two), "v"(w));
    if (B == 2) asm("v_lshlrev_b32_sdwa %0, %1, %2 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:BYTE_2" : "=v"(r) : "v"(two), "v"(w));
    if (B == 3) asm("v_lshlrev_b32_sdwa %0, %1, %2 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:BYTE_3" : "=v"(r) : "v"(two), "v"(w));
    return r;
}

// acc + sum_m T[m][byte m of the word] for the four bytes of one code word,
// sub-quantisers m0 .. m0+3; T is the table base as a byte pointer.
template <int M0>
__device__ __forceinline__ float adc_word(uint32_t w, const char *T, float acc, uint32_t two)
{
    acc += *reinterpret_cast<const float *>(T + (M0 + 0) * 1024 + byte_x4<0>(w, two));
    acc += *reinterpret_cast<const float *>(T + (M0 + 1) * 1024 + byte_x4<1>(w, two));
    acc += *reinterpret_cast<const float *>(T + (M0 + 2) * 1024 + byte_x4<2>(w, two));
    acc += *reinterpret_cast<const float *>(T + (M0 + 3) * 1024 + byte_x4<3>(w, two));
    return acc;
}

template <int M>
__device__ __forceinline__ float adc_sum(const typename CodeWord<M>::type &c, const char *T, float acc, uint32_t two);

template <>
__device__ __forceinline__ float adc_sum<16>(const u32x4 &c, const char *T, float acc, uint32_t two)
{
    acc = adc_word<0>(c.x, T, acc, two);
    acc = adc_word<4>(c.y, T, acc, two);
    acc = adc_word<8>(c.z, T, acc, two);
    return adc_word<12>(c.w, T, acc, two);
}

template <>
__device__ __forceinline__ float adc_sum<8>(const u32x2 &c, const char *T, float acc, uint32_t two)
{
    acc = adc_word<0>(c.x, T, acc, two);
    return adc_word<4>(c.y, T, acc, two);
}

// Sort the wave's pool, keep its k best, return the new admission threshold
// (any pool capacity; used when the pool does not fit the register path below).
__device__ __forceinline__ float wave_pool_sort(uint64_t *pool, int cap, int &pool_n, int k)
{
    const int lane = threadIdx.x & (WAVE - 1);
    for (int i = pool_n + lane; i < cap; i += WAVE) pool[i] = EMPTY_KEY;
    wave_bitonic_sort(pool, cap);
    if (pool_n > k) pool_n = k;
    float theta = INFINITY;
    if (pool_n == k) theta = key_float((uint32_t)(pool[k - 1] >> 32));
    return theta;
}

// The same for a pool of 256 keys without sorting: four keys per lane in
// registers, the k-th smallest found by an MSB-first bitwise search with
// wave-wide population counts (first over the distance word; over the low word
// only when distances tie at the boundary), survivors written back compacted
// (unordered).  Exactly min(pool_n, k) keys survive.
__device__ __forceinline__ float wave_pool_select256(uint64_t *pool, int &pool_n, int k)
{
    if (pool_n <= k) return INFINITY;
    const int lane = threadIdx.x & (WAVE - 1);
    uint32_t hi[4], lo[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int idx = lane + WAVE * j;
        const uint64_t key = idx < pool_n ? pool[idx] : EMPTY_KEY;
        hi[j] = (uint32_t)(key >> 32);
        lo[j] = (uint32_t)key;
    }
    uint32_t pref = 0;
    int rem = k;
    for (int bit = 31; bit >= 0; --bit) {
        const uint32_t mask = ~((1u << bit) - 1u);
        int cnt = 0;
#pragma unroll
        for (int j = 0; j < 4; ++j) cnt += __popcll(__ballot((hi[j] & mask) == pref));
        if (rem > cnt) { rem -= cnt; pref |= 1u << bit; }
    }
    int ceq = 0;
#pragma unroll
    for (int j = 0; j < 4; ++j) ceq += __popcll(__ballot(hi[j] == pref));
    uint32_t lo_thr = 0xFFFFFFFFu;
    if (ceq > rem) {   // equal distances straddle rank k: keep the rem lowest low words
        uint32_t p2 = 0;
        int r2 = rem;
        for (int bit = 31; bit >= 0; --bit) {
            const uint32_t mask = ~((1u << bit) - 1u);
            int cnt = 0;
#pragma unroll
            for (int j = 0; j < 4; ++j) cnt += __popcll(__ballot(hi[j] == pref && (lo[j] & mask) == p2));
            if (r2 > cnt) { r2 -= cnt; p2 |= 1u << bit; }
        }
        lo_thr = p2;
    }
    wave_sync();
    int base = 0;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const bool keep = hi[j] < pref || (hi[j] == pref && lo[j] <= lo_thr);
        const uint64_t m = __ballot(keep);
        if (keep) pool[base + __popcll(m & ((1ull << lane) - 1ull))] = ((uint64_t)hi[j] << 32) | lo[j];
        base += __popcll(m);
    }
    pool_n = base;
    wave_sync();
    return key_float(pref);
}

__device__ __forceinline__ float wave_pool_compact(uint64_t *pool, int cap, int &pool_n, int k)
{
    return cap == 256 ? wave_pool_select256(pool, pool_n, k) : wave_pool_sort(pool, cap, pool_n, k);
}

constexpr int SCAN_U = 4;                     // 64-record steps per chunk
constexpr int SCAN_CHUNK = WAVE * SCAN_U;     // records a wavefront has in flight per chunk

// Per-wavefront LDS staging of a batch of 64 descriptors.
struct WaveStage {
    // the batch's non-empty descriptors, compacted in order:
    uint4 a[WAVE];              // address of the codes (lo, hi), address of the constant bytes (lo, hi)
    uint4 b[WAVE];              // first flattened record index, len, base (bits), pos0
    uint8_t mark[SCAN_CHUNK];   // 1 where the first record of a descriptor sits, else 0
};
static_assert(SCAN_CHUNK % 16 == 0 && sizeof(WaveStage) % 16 == 0, "stage arrays must stay 16-byte aligned");

template <int M>
struct ChunkRegs {
    typename CodeWord<M>::type code[SCAN_U];
    uint32_t cb[SCAN_U];        // constant byte
    float base[SCAN_U];
    uint32_t c[SCAN_U];         // grouped position of the record (indexes ids[]); 0xFFFFFFFF = no record
};

// Find the owner of every record of the chunk starting at flattened index t0
// and issue its two loads.  Every lane issues both loads of every step whatever
// T is (lanes without a record read the address held in slot 0 of the stage),
// so the number of loads in flight is the same on every path and a chunk can
// be waited for while the one issued after it is still outstanding.
template <int M>
__device__ __forceinline__ void scan_issue(ChunkRegs<M> &r, WaveStage &st, uint32_t t0, uint32_t T,
                                           uint32_t len, uint32_t pre, uint32_t &carry)
{
    typedef typename CodeWord<M>::type code_t;
    const int lane = threadIdx.x & (WAVE - 1);
#pragma unroll
    for (int i = lane; i < SCAN_CHUNK / 4; i += WAVE) reinterpret_cast<uint32_t *>(st.mark)[i] = 0u;
    wave_sync();
    if (len > 0 && pre >= t0 && pre - t0 < (uint32_t)SCAN_CHUNK) st.mark[pre - t0] = 1;
    wave_sync();
    // The owner of record t is the descriptor whose head is the last one at or before t.  The
    // stage holds the non-empty descriptors in order, so its slot is (number of heads at or
    // before t) - 1: heads before this 64-record step (carry, wave-uniform), plus heads at
    // lower lanes of the step (population count of the ballot below the lane), plus its own.
    uint32_t head[SCAN_U];
#pragma unroll
    for (int u = 0; u < SCAN_U; ++u) head[u] = (uint32_t)st.mark[WAVE * u + lane];
#pragma unroll
    for (int u = 0; u < SCAN_U; ++u) {
        const uint32_t t = t0 + WAVE * u + lane;
        const uint64_t hm = __ballot(head[u] != 0);
        const uint32_t below = __builtin_amdgcn_mbcnt_hi((uint32_t)(hm >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)hm, 0u));
        const uint32_t o = carry + below + head[u];
        carry += (uint32_t)__popcll(hm);
        bool act = t < T && o > 0;
        const uint32_t oi = act ? (o - 1) & (WAVE - 1) : 0;   // always inside the stage
        const uint4 db = st.b[oi];
        const uint4 da = st.a[oi];
        uint32_t c = t - db.x;
        act = act && c < db.y;                     // never read outside the owner's block
        c = act ? c : 0u;
        r.c[u] = act ? db.w + c : 0xFFFFFFFFu;
        r.base[u] = __uint_as_float(db.z);
        typedef const __attribute__((address_space(1))) code_t *gcode_p;   // global, not flat, loads
        typedef const __attribute__((address_space(1))) uint8_t *gbyte_p;
        const uint64_t pc = ((uint64_t)da.y << 32) | da.x, pb = ((uint64_t)da.w << 32) | da.z;
        r.code[u] = *reinterpret_cast<gcode_p>(pc + (uint64_t)c * M);
        r.cb[u] = *reinterpret_cast<gbyte_p>(pb + c);
    }
}

// Grid: nq * nsplit workgroups; workgroup (q, split) scans an equal share of
// the query's S descriptors, each wavefront batches of 64 of them.  The
// records of a batch are flattened: a prefix sum of the lengths numbers them,
// every lane takes record t = t0 + 64u + lane of the current chunk, and finds
// the owning descriptor from head marks in LDS by counting the heads before it
// (ballot + population count).  All lanes are busy whatever the subregion lengths, a
// 16-byte code is one 128-bit load, and the loads of the next chunk are issued
// before the table lookups of the current one, so each wavefront keeps two
// chunks (about 8 KB) in flight.  The M bytes index the query's table in LDS;
// the estimate (Eq. (6)) is offered to the wavefront's top-k pool, keyed by
// (distance, grouped position): ids are not touched here, the final k-select
// reads them for the survivors and orders by (distance, id).  The admission
// threshold is shared by the workgroup's wavefronts: once any of them holds k
// candidates, nothing above its k-th distance can be a result.
// Output: per (q, split, wave) the k best keys (distance, position), in no
// particular order, padded with EMPTY_KEY.
template <int M>
__global__ __launch_bounds__(SCAN_BLOCK) __attribute__((amdgpu_waves_per_eu(4, 4))) void scan_kernel(
    const uint8_t *__restrict__ blocks, const float *__restrict__ const_table,
    const SubDesc *__restrict__ desc, int S, const float *__restrict__ lut, int k, int nsplit,
    uint64_t *__restrict__ partial)
{
    // The table sits in static LDS so that its address is a compile-time constant and every
    // lookup is one ds_read with an immediate offset; only the pools are sized at launch.
    __shared__ __attribute__((aligned(16))) float T[M * 256];
    __shared__ float nt[256];
    __shared__ WaveStage stages[SCAN_WAVES];
    __shared__ uint32_t wg_theta_key;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    uint64_t *pools = reinterpret_cast<uint64_t *>(smem);                  // SCAN_WAVES * cap

    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int64_t q = blockIdx.x / nsplit;
    const int split = blockIdx.x % nsplit;
    const int cap = pool_capacity(k);
    uint64_t *pool = pools + wave * cap;
    WaveStage &st = stages[wave];
    const char *Tb = reinterpret_cast<const char *>(T);
    uint32_t two = 2;
    asm volatile("" : "+v"(two));   // keep the shift amount in a vector register

    {
        const float4 *src = reinterpret_cast<const float4 *>(lut + q * (int64_t)(M * 256));
        float4 *dst = reinterpret_cast<float4 *>(T);
        for (int i = tid; i < M * 64; i += SCAN_BLOCK) dst[i] = src[i];
        nt[tid] = const_table[tid];
        if (tid == 0) wg_theta_key = float_key(INFINITY);
    }
    __syncthreads();

    const int d_begin = (int)(((int64_t)S * split) / nsplit);
    const int d_end = (int)(((int64_t)S * (split + 1)) / nsplit);
    const SubDesc *qd = desc + q * S;

    int pool_n = 0;
    float theta = INFINITY;

    // The wavefront's descriptors form one stream of chunks that runs across batch boundaries:
    // next() stages the next batch when the current one is exhausted (the stage is only read
    // while issuing) and issues the following chunk into the given register set.
    // Slot 0 of the stage always holds a readable address: the query's table until the first
    // non-empty descriptor is staged.
    if (lane == 0) {
        const uint64_t dummy = reinterpret_cast<uint64_t>(lut + q * (int64_t)(M * 256));
        st.a[0] = make_uint4((uint32_t)dummy, (uint32_t)(dummy >> 32), (uint32_t)dummy, (uint32_t)(dummy >> 32));
        st.b[0] = make_uint4(0u, 0u, 0u, 0u);
    }
    wave_sync();
    if (d_begin >= d_end) {                       // nothing kept (wave-uniform)
        uint64_t *o = partial + ((q * nsplit + split) * SCAN_WAVES + wave) * (int64_t)k;
        for (int i = lane; i < k; i += WAVE) o[i] = EMPTY_KEY;
        return;
    }
    // Descriptor prefetch: always one load per lane (index clamped into the share), validity
    // is applied when the batch is staged.
    int b_next = d_begin + wave * WAVE;          // first descriptor of the batch to stage next
    auto fetch_desc = [&](int b) {
        int i = b + lane;
        i = i < d_end ? i : d_end - 1;
        return *reinterpret_cast<const uint4 *>(qd + i);
    };
    uint4 sd_next = fetch_desc(b_next);
    uint32_t len = 0, pre = 0, Tn = 0, t_next = 0, carry = 0;
    auto stage = [&]() {
        const uint4 sd = sd_next;                 // blk, pos0, len, base
        const bool valid = b_next + lane < d_end;
        b_next += SCAN_WAVES * WAVE;
        sd_next = fetch_desc(b_next);             // prefetch the batch after (b_next may pass d_end: clamped)
        len = valid ? sd.z : 0u;
        const uint32_t inc = wave_inclusive_scan(len);
        pre = inc - len;
        Tn = (uint32_t)__builtin_amdgcn_readlane((int)inc, WAVE - 1);
        t_next = 0;
        carry = 0;
        wave_sync();
        const uint64_t pc = reinterpret_cast<uint64_t>(blocks) + (uint64_t)sd.x * (uint64_t)BLK_ALIGN;
        const uint64_t pb = pc + (uint64_t)len * M;
        const uint64_t ne = __ballot(len > 0);
        const uint32_t slot = __builtin_amdgcn_mbcnt_hi((uint32_t)(ne >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)ne, 0u));
        if (len > 0) {
            st.a[slot] = make_uint4((uint32_t)pc, (uint32_t)(pc >> 32), (uint32_t)pb, (uint32_t)(pb >> 32));
            st.b[slot] = make_uint4(pre, len, sd.w, sd.y);
        }
    };
    // Issues the next chunk of the stream into r; when the stream has ended it still issues a
    // chunk of loads with no records (so that load counts do not depend on the path taken) and
    // returns false.
    auto next = [&](ChunkRegs<M> &r) -> bool {
        bool live = true;
        while (t_next >= Tn) {                    // current batch exhausted (or empty): stage the next one
            if (b_next >= d_end) { live = false; break; }
            stage();
        }
        scan_issue<M>(r, st, t_next, live ? Tn : 0u, live ? len : 0u, pre, carry);
        t_next += SCAN_CHUNK;
        return live;
    };
    // Table lookups of the whole chunk first, as one straight run of code for all lanes (lanes
    // without a record look up the bytes their placeholder load returned and are masked out
    // afterwards): the 4 * (M + 1) LDS reads and the four sums are independent and overlap.
    // Admission to the pool is rare once the threshold has tightened and is tested once per chunk.
    auto consume = [&](ChunkRegs<M> &cur) {
        theta = fminf(theta, key_float(wg_theta_key));
        float dist[SCAN_U];
#pragma unroll
        for (int u = 0; u < SCAN_U; ++u)
            dist[u] = adc_sum<M>(cur.code[u], Tb, cur.base[u] + nt[cur.cb[u]], two);
        bool any = false;
#pragma unroll
        for (int u = 0; u < SCAN_U; ++u) any = any || (cur.c[u] != 0xFFFFFFFFu && dist[u] <= theta);
        if (__ballot(any) == 0) return;
#pragma nounroll
        for (int u = 0; u < SCAN_U; ++u) {        // rolled: one copy of the rarely taken path
            float d = dist[0];
            uint32_t c = cur.c[0];
#pragma unroll
            for (int j = 1; j < SCAN_U; ++j) {
                d = u == j ? dist[j] : d;
                c = u == j ? cur.c[j] : c;
            }
            const bool pass = c != 0xFFFFFFFFu && d <= theta;
            const uint64_t mask = __ballot(pass);
            if (mask) {
                if (pass) {
                    int slot = pool_n + __popcll(mask & ((1ull << lane) - 1ull));
                    pool[slot] = ((uint64_t)float_key(d) << 32) | c;
                }
                pool_n += __popcll(mask);
                if (pool_n > cap - WAVE) {
                    theta = wave_pool_compact(pool, cap, pool_n, k);
                    if (lane == 0) atomicMin(&wg_theta_key, float_key(theta));
                }
            }
        }
    };
    // two register sets used alternately: the loads of chunk c+1 are in flight while chunk c is consumed
    ChunkRegs<M> ra, rb;
    bool va = next(ra);
    while (va) {
        const bool vb = next(rb);
        consume(ra);
        if (!vb) break;
        va = next(ra);
        consume(rb);
    }
    wave_pool_compact(pool, cap, pool_n, k);
    uint64_t *out = partial + ((q * nsplit + split) * SCAN_WAVES + wave) * (int64_t)k;
    for (int i = lane; i < k; i += WAVE) out[i] = i < pool_n ? pool[i] : EMPTY_KEY;
}

// Final k-select: replace the position of every partial key by the point's id and write the k
// best of a query's n_in keys by (distance, id); empty slots become (-1, +inf).  Two steps: a
// radix select on the distance word finds the k-th smallest distance, then only the keys at or
// below it (k of them, plus ties on that distance) are sorted, instead of all n_in.
// Dynamic LDS: (n_in + n_pow2) keys, n_pow2 = next power of two of n_in.
template <int BLOCK>
__global__ __launch_bounds__(BLOCK) void merge_kernel(const uint64_t *__restrict__ partial,
                                                      const int32_t *__restrict__ ids, int n_in,
                                                      int n_pow2, int k, int32_t *__restrict__ out_ids,
                                                      float *__restrict__ out_dists)
{
    __shared__ SelectShared sh;
    __shared__ uint32_t cnt_s;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    uint64_t *a = reinterpret_cast<uint64_t *>(smem);      // n_in gathered keys
    uint64_t *b = a + n_in;                                // the selected ones, sorted
    const int64_t q = blockIdx.x;
    uint32_t have = 0;
    for (int i = threadIdx.x; i < n_in; i += BLOCK) {
        uint64_t key = partial[q * n_in + i];
        if (key != EMPTY_KEY) {
            key = (key & 0xFFFFFFFF00000000ull) | (uint32_t)ids[(uint32_t)key];
            ++have;
        }
        a[i] = key;
    }
    uint32_t n_valid;
    block_exclusive_scan<BLOCK>(have, sh.scan, n_valid);   // contains barriers: a[] is complete
    uint32_t pivot = 0xFFFFFFFFu, need = 0;
    auto hi = [a](int64_t i) { return (uint32_t)(a[i] >> 32); };
    if (n_valid > (uint32_t)k) block_radix_select<BLOCK>(hi, n_in, (uint32_t)k, sh, pivot, need);   // uniform branch
    // keys with distance <= pivot, in any order (ties on the pivot distance are all kept: the sort decides by id)
    if (threadIdx.x == 0) cnt_s = 0;
    __syncthreads();
    for (int i = threadIdx.x; i < n_in; i += BLOCK) {
        const uint64_t key = a[i];
        if (key != EMPTY_KEY && (uint32_t)(key >> 32) <= pivot) b[atomicAdd(&cnt_s, 1u)] = key;
    }
    __syncthreads();
    const int m = (int)cnt_s;
    int mp = 1;
    while (mp < m) mp <<= 1;
    for (int i = m + threadIdx.x; i < mp; i += BLOCK) b[i] = EMPTY_KEY;
    block_bitonic_sort<BLOCK>(b, mp);
    for (int i = threadIdx.x; i < k; i += BLOCK) {
        uint64_t key = i < m ? b[i] : EMPTY_KEY;
        bool empty = key == EMPTY_KEY;
        out_ids[q * k + i] = empty ? -1 : (int32_t)(uint32_t)key;
        out_dists[q * k + i] = empty ? INFINITY : key_float((uint32_t)(key >> 32));
    }
}

}  // namespace ivf
