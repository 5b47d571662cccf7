// C ABI of the library (see include/ivf_gp.h): argument checks, scratch
// management and the launch sequence of the query path.  gfx950 only.
#include "../../include/ivf_gp.h"

#include <atomic>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <new>
#include <string>
#include <vector>

#include <hip/hip_runtime.h>
#include <rocprim/device/device_scan.hpp>

#include "budget.hpp"
#include "coarse.hpp"
#include "encode.hpp"
#include "latency.hpp"
#include "layout.hpp"
#include "query.hpp"
#include "scan.hpp"
#include "train.hpp"

using namespace ivf;

namespace {

thread_local std::string g_err;

int fail(int code, const char *fmt, ...)
{
    char buf[512];
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(buf, sizeof buf, fmt, ap);
    va_end(ap);
    g_err = buf;
    return code;
}

#define HIPCHK(expr)                                                                         \
    do {                                                                                     \
        hipError_t e_ = (expr);                                                              \
        if (e_ != hipSuccess)                                                                \
            return fail(e_ == hipErrorOutOfMemory ? IVF_ENOMEM : IVF_EHIP, "%s: %s", #expr,  \
                        hipGetErrorString(e_));                                              \
    } while (0)

#define LAUNCHCHK(name)                                                                      \
    do {                                                                                     \
        hipError_t e_ = hipGetLastError();                                                   \
        if (e_ != hipSuccess) return fail(IVF_EHIP, "launch %s: %s", name, hipGetErrorString(e_)); \
    } while (0)

struct Buf {
    void *p = nullptr;
    size_t bytes = 0;
};

// device memory released when the scope ends, error returns included (the owner synchronizes first)
struct DevTmp {
    void *p = nullptr;
    DevTmp() = default;
    DevTmp(const DevTmp &) = delete;
    DevTmp &operator=(const DevTmp &) = delete;
    ~DevTmp() { if (p) (void)hipFree(p); }
};

int ensure(Buf &b, size_t bytes)
{
    if (bytes <= b.bytes) return IVF_OK;
    if (b.p) {
        HIPCHK(hipDeviceSynchronize());
        HIPCHK(hipFree(b.p));
        b.p = nullptr;
        b.bytes = 0;
    }
    HIPCHK(hipMalloc(&b.p, bytes));
    b.bytes = bytes;
    return IVF_OK;
}

bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

int next_pow2(int v)
{
    int p = 1;
    while (p < v) p <<= 1;
    return p;
}

int check_trained(const ivf_index_desc *d)
{
    if (!d) return fail(IVF_EINVAL, "index descriptor is NULL");
    if (d->D < 4 || d->D > IVF_MAX_D || d->D % 4) return fail(IVF_EINVAL, "D=%d must be a multiple of 4 in [4, %d]", d->D, IVF_MAX_D);
    if (d->M != 8 && d->M != 16) return fail(IVF_EINVAL, "M=%d must be 8 or 16", d->M);
    if (d->D % d->M) return fail(IVF_EINVAL, "D=%d is not a multiple of M=%d", d->D, d->M);
    if (d->L < 1 || d->K < 1) return fail(IVF_EINVAL, "K=%lld and L=%d must be positive", (long long)d->K, d->L);
    if ((int64_t)d->L >= d->K && d->K > 1) return fail(IVF_EINVAL, "L=%d needs at least L+1 centroids", d->L);
    if (d->K * (int64_t)d->L >= (1ll << 31)) return fail(IVF_EINVAL, "K*L must be below 2^31");
    if (!d->centroids || !d->nbr || !d->alpha || !d->cs_dist2)
        return fail(IVF_EINVAL, "a trained array (centroids, nbr, alpha, cs_dist2) is NULL");
    if (!aligned16(d->centroids)) return fail(IVF_EINVAL, "centroids must be 16-byte aligned");
    return IVF_OK;
}

// ------------------------------------------------------------ stage 1 driver
// Packs the rows of X for the GEMM (hi/lo fp16 stages, see split_rows_kernel) and writes their
// squared norms and inverse scales.  gmax != NULL: one scale for the whole matrix (gmax is a
// device word used for the reduction, inv receives one float); else one scale per row.
int pack_rows(const float *X, int64_t n, int D, uint32_t *gmax, _Float16 *P, float *norm, float *inv,
              hipStream_t st)
{
    if (n <= 0) return IVF_OK;
    if (gmax) {
        HIPCHK(hipMemsetAsync(gmax, 0, sizeof(uint32_t), st));
        const int64_t count = n * D;
        int64_t grid = (count + 255) / 256;
        if (grid > 16384) grid = 16384;
        absmax_kernel<<<dim3((unsigned)grid), dim3(256), 0, st>>>(X, count, gmax);
        LAUNCHCHK("absmax_kernel");
    }
    split_rows_kernel<<<dim3((unsigned)((n + 3) / 4)), dim3(256), 0, st>>>(X, n, D, gmax, P, norm, inv);
    LAUNCHCHK("split_rows_kernel");
    return IVF_OK;
}

int launch_coarse(const _Float16 *xp, const float *xn, const float *xsi, int64_t nq, const _Float16 *Cp,
                  const float *cn, const float *csi, int64_t K, int Dp, float *Dt, float *bm, hipStream_t st)
{
    const int64_t ldt = dt_stride(K);
    const int nb = (int)((K + BMW - 1) / BMW);
    if (nq <= 2 * SKQ) {   // small batch: one tile of 32 or 64 queries, the centroid table streamed once
        const int64_t cblocks = (K + SKC - 1) / SKC;
        const int64_t grid = (cblocks + N_XCD - 1) / N_XCD * N_XCD;
        if (nq <= SKQ)
            coarse_gemm_skinny_kernel<1><<<dim3((unsigned)grid), dim3(256), 0, st>>>(xp, xn, xsi, nq, Cp, cn, csi, K, Dp, Dt, ldt, bm, nb, 1);
        else
            coarse_gemm_skinny_kernel<2><<<dim3((unsigned)grid), dim3(256), 0, st>>>(xp, xn, xsi, nq, Cp, cn, csi, K, Dp, Dt, ldt, bm, nb, 1);
        LAUNCHCHK("coarse_gemm_skinny_kernel");
        return IVF_OK;
    }
    int tiles_q = (int)((nq + GT - 1) / GT);
    int64_t tiles_c = (K + GT - 1) / GT;
    int64_t grid = (int64_t)((tiles_q + N_XCD - 1) / N_XCD) * N_XCD * tiles_c;
    if (grid >= (1ll << 24)) return fail(IVF_EINVAL, "coarse tile grid too large (more than 2^32 threads)");
    const int stages = Dp / DK;
    if ((stages == 6 || stages == 8) && K % GT == 0) {
        // Query tile held in registers, centroid tiles swept.  The kernel works on whole tiles: the
        // rows of a partial last query tile are computed too, into the padding every per-query
        // buffer of the coarse stage carries up to a multiple of the tile height.
        const int per_wg = 64;
        static_assert(per_wg % SWEEP_BMC == 0, "a workgroup's first tile starts a 64-byte piece of the block minima");
        const int64_t groups = (tiles_c + per_wg - 1) / per_wg;
        const int64_t g2 = (int64_t)((tiles_q + N_XCD - 1) / N_XCD) * N_XCD * groups;
        if (g2 >= (1ll << 24)) return fail(IVF_EINVAL, "coarse tile grid too large (more than 2^32 threads)");
        if (stages == 6)
            coarse_gemm_sweep_kernel<6><<<dim3((unsigned)g2), dim3(256), 0, st>>>(xp, xn, xsi, (int64_t)tiles_q * GT, Cp, cn, csi, K, Dt, ldt, bm, nb, tiles_q, (int)tiles_c, per_wg);
        else
            coarse_gemm_sweep_kernel<8><<<dim3((unsigned)g2), dim3(256), 0, st>>>(xp, xn, xsi, (int64_t)tiles_q * GT, Cp, cn, csi, K, Dt, ldt, bm, nb, tiles_q, (int)tiles_c, per_wg);
        LAUNCHCHK("coarse_gemm_sweep_kernel");
        return IVF_OK;
    }
    coarse_gemm_kernel<<<dim3((unsigned)grid), dim3(256), 0, st>>>(xp, xn, xsi, nq, Cp, cn, csi, K, Dp, Dt, ldt, bm, nb, tiles_q);
    LAUNCHCHK("coarse_gemm_kernel");
    return IVF_OK;
}

int launch_probe_select(const float *Dt, const float *bm, int64_t nq, int64_t K, int P, int32_t *pid,
                        float *pd, hipStream_t st)
{
    const int nb = (int)((K + BMW - 1) / BMW);
    const size_t lds = (size_t)2 * P * sizeof(int);
    if (P <= PS_P_MAX && nb <= PS_NB_MAX) {   // keys in LDS
        const size_t lds2 = ((size_t)2 * P + 3 + (nb > 2 * PS_CAP ? nb : 2 * PS_CAP)) * sizeof(int);
        if (lds2 > 48 * 1024)
            HIPCHK(hipFuncSetAttribute(reinterpret_cast<const void *>(&probe_select_lds_kernel),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds2));
        probe_select_lds_kernel<<<dim3((unsigned)nq), dim3(1024), lds2, st>>>(Dt, dt_stride(K), bm, K, nb, P, pid, pd);
        LAUNCHCHK("probe_select_lds_kernel");
        return IVF_OK;
    }
    if (P >= 1024)
        probe_select_kernel<1024><<<dim3((unsigned)nq), dim3(1024), lds, st>>>(Dt, dt_stride(K), bm, K, nb, P, pid, pd);
    else
        probe_select_kernel<256><<<dim3((unsigned)nq), dim3(256), lds, st>>>(Dt, dt_stride(K), bm, K, nb, P, pid, pd);
    LAUNCHCHK("probe_select_kernel");
    return IVF_OK;
}

// Device scratch of one pass over a tile of queries, and the launch shape that goes with it.
struct SearchWs {
    float *dt = nullptr, *bm = nullptr, *qn = nullptr, *qsi = nullptr;
    _Float16 *qpk = nullptr;
    int32_t *probe_id = nullptr;
    float *probe_d = nullptr;
    SubDesc *desc = nullptr;
    float *lut = nullptr;
    uint64_t *partial = nullptr;
    float *qrot = nullptr;       // rotated queries (indexes with a rotation in front of the PQ)
};

enum { WS_DT, WS_BM, WS_QN, WS_QSI, WS_QPK, WS_PID, WS_PD, WS_DESC, WS_LUT, WS_PARTIAL, WS_QROT, WS_COUNT };

struct SearchPlan {
    int64_t tile = 0;            // queries per pass
    int S = 0, nsplit = 1, n_lists = 0, merge_n = 0, merge_pow2 = 0;
    size_t bytes[WS_COUNT] = {};
};

// Rows of the distance tile (and of the block minima) a pass over n queries may write: the sweep
// kernel works on whole tiles of GT query rows, the other two check every row.
int64_t dt_rows(int64_t n, int64_t K, int Dp)
{
    const int stages = Dp / DK;
    const bool sweep = n > 2 * SKQ && (stages == 6 || stages == 8) && K % GT == 0;
    return sweep ? (n + GT - 1) / GT * GT : n;
}

SearchPlan plan_search(int64_t K, int D, int M, int P, int S, int k, int64_t tile, bool rotated)
{
    SearchPlan pl;
    pl.tile = tile;
    pl.S = S;
    // workgroups per query in the scan: fill the chip when the batch is small, but with at most 8 per
    // query: every workgroup hands 4 k candidates to the final k-select, whose time grows with them
    // faster than the scan's shrinks (one query on the 100M-point workload, scan + k-select in us:
    // 17 + 9 with 2 workgroups, 12 + 9 with 4, 10.5 + 10 with 8, 10 + 12 / 14 / 20 with 16 / 32 / 64)
    int nsplit = (int)((2048 + tile - 1) / tile);
    if (nsplit > 8) nsplit = 8;
    if (nsplit > (S + 15) / 16) nsplit = (S + 15) / 16;
    while (nsplit > 1 && (int64_t)nsplit * SCAN_WAVES * k > 8192) --nsplit;
    if (nsplit < 1) nsplit = 1;
    pl.nsplit = nsplit;
    pl.n_lists = nsplit * SCAN_WAVES;
    pl.merge_n = pl.n_lists * k;
    pl.merge_pow2 = next_pow2(pl.merge_n);
    const int Dp = packed_dim(D);
    const size_t rows = (size_t)dt_rows(tile, K, Dp);
    const size_t tile_pad = (size_t)packed_rows(tile);   // the GEMM tiles copy whole tiles of packed rows
    const int64_t nb = (K + BMW - 1) / BMW;
    pl.bytes[WS_DT] = rows * dt_stride(K) * sizeof(float);
    pl.bytes[WS_BM] = rows * nb * sizeof(float);
    pl.bytes[WS_QN] = tile_pad * sizeof(float);
    pl.bytes[WS_QSI] = tile_pad * sizeof(float);
    pl.bytes[WS_QPK] = tile_pad * Dp * 2 * sizeof(_Float16);
    pl.bytes[WS_PID] = (size_t)tile * P * sizeof(int32_t);
    pl.bytes[WS_PD] = (size_t)tile * P * sizeof(float);
    pl.bytes[WS_DESC] = (size_t)tile * S * sizeof(SubDesc);
    pl.bytes[WS_LUT] = (size_t)tile * M * 256 * sizeof(float);
    pl.bytes[WS_PARTIAL] = (size_t)tile * pl.merge_n * sizeof(uint64_t);
    pl.bytes[WS_QROT] = rotated ? (size_t)tile * D * sizeof(float) : 0;
    return pl;
}

}  // namespace

struct ivf_index {
    int D = 0, M = 0, L = 0;
    int64_t K = 0, N = 0;
    float *centroids = nullptr, *cnorm = nullptr, *alpha = nullptr, *cst = nullptr;
    _Float16 *cpk = nullptr;     // centroids packed for the GEMM
    float *csi = nullptr;        // csi[0] inverse scale of the packed centroids; csi[1] reduction word
    float *codebook = nullptr, *const_table = nullptr;
    float *rot_t = nullptr;      // transposed rotation in front of the PQ, or NULL
    int32_t *nbr = nullptr, *ids = nullptr;
    uint4 *sub_info = nullptr;   // per subregion: block offset, first position, length
    uint8_t *blocks = nullptr;
    int64_t scratch_limit = 8ll << 30;
    Buf dt, bm, qn, qpk, qsi, probe_id, probe_d, desc, lut, partial, qrot;
    // optional per-stage timing with HIP events on the caller's stream
    bool profile = false;
    std::vector<hipEvent_t> ev[IVF_N_STAGES + 1];   // ev[s][i], ev[s+1][i] bracket stage s of pass i
    int64_t launches = 0;
};

extern "C" const char *ivf_last_error(void) { return g_err.c_str(); }

extern "C" int64_t ivf_num_kept(int nprobe, int L, float prune_frac)
{
    int64_t total = (int64_t)nprobe * L;
    int64_t S = (int64_t)std::ceil((double)prune_frac * (double)nprobe * (double)L);
    if (S < 1) S = 1;
    if (S > total) S = total;
    return S;
}

extern "C" void ivf_free_index(ivf_index *ix)
{
    if (!ix) return;
    (void)hipDeviceSynchronize();
    void *owned[] = {ix->centroids, ix->cnorm, ix->alpha, ix->cst, ix->codebook, ix->const_table,
                     ix->nbr, ix->ids, ix->sub_info, ix->blocks, ix->dt.p, ix->bm.p, ix->qn.p,
                     ix->cpk, ix->csi, ix->qpk.p, ix->qsi.p,
                     ix->probe_id.p, ix->probe_d.p, ix->desc.p, ix->lut.p, ix->partial.p, ix->qrot.p, ix->rot_t};
    for (void *p : owned)
        if (p) (void)hipFree(p);
    for (auto &v : ix->ev)
        for (hipEvent_t e : v) (void)hipEventDestroy(e);
    delete ix;
}

extern "C" int ivf_set_scratch_limit(ivf_index *ix, int64_t bytes)
{
    if (!ix || bytes < 4096) return fail(IVF_EINVAL, "scratch limit must be at least 4096 bytes");
    ix->scratch_limit = bytes;
    return IVF_OK;
}

namespace {

template <class T>
int dev_copy(T *&dst, const T *src, size_t count, hipStream_t st)
{
    HIPCHK(hipMalloc(reinterpret_cast<void **>(&dst), count * sizeof(T) ? count * sizeof(T) : 16));
    if (count) HIPCHK(hipMemcpyAsync(dst, src, count * sizeof(T), hipMemcpyDeviceToDevice, st));
    return IVF_OK;
}

int load_impl(const ivf_index_desc *d, hipStream_t st, ivf_index *ix)
{
    const int64_t K = d->K, N = d->N, nsub = K * d->L;
    const int D = d->D, M = d->M, L = d->L;
    ix->D = D; ix->M = M; ix->L = L; ix->K = K; ix->N = N;
    int rc;
    if ((rc = dev_copy(ix->centroids, d->centroids, (size_t)K * D, st))) return rc;
    if ((rc = dev_copy(ix->nbr, d->nbr, (size_t)nsub, st))) return rc;
    if ((rc = dev_copy(ix->alpha, d->alpha, (size_t)K, st))) return rc;
    if ((rc = dev_copy(ix->codebook, d->pq_codebook, (size_t)256 * D, st))) return rc;
    if ((rc = dev_copy(ix->const_table, d->const_table, (size_t)256, st))) return rc;
    if ((rc = dev_copy(ix->ids, d->ids, (size_t)N, st))) return rc;

    if (d->rotation) {
        HIPCHK(hipMalloc(reinterpret_cast<void **>(&ix->rot_t), (size_t)D * D * sizeof(float)));
        transpose_square_kernel<<<dim3((unsigned)((D * D + 255) / 256)), dim3(256), 0, st>>>(d->rotation, D, ix->rot_t);
        LAUNCHCHK("transpose_square_kernel");
    }
    HIPCHK(hipMalloc(reinterpret_cast<void **>(&ix->cnorm), (size_t)K * sizeof(float)));
    HIPCHK(hipMalloc(reinterpret_cast<void **>(&ix->cpk), (size_t)packed_rows(K) * packed_dim(D) * 2 * sizeof(_Float16)));
    HIPCHK(hipMalloc(reinterpret_cast<void **>(&ix->csi), 2 * sizeof(float)));
    if ((rc = pack_rows(ix->centroids, K, D, reinterpret_cast<uint32_t *>(ix->csi + 1), ix->cpk, ix->cnorm, ix->csi, st)))
        return rc;
    HIPCHK(hipMalloc(reinterpret_cast<void **>(&ix->cst), (size_t)nsub * sizeof(float)));
    cst_kernel<<<dim3((unsigned)((nsub + 255) / 256)), dim3(256), 0, st>>>(ix->alpha, d->cs_dist2, L, nsub, ix->cst);
    LAUNCHCHK("cst_kernel");

    // 64-bit check of the 32-bit block offsets: N*(M+1) bytes plus at most one block of padding each
    if (((uint64_t)N * (M + 1)) / BLK_ALIGN + (uint64_t)nsub >= (1ull << 32))
        return fail(IVF_EINVAL, "index too large for 32-bit block offsets");
    // block offsets: exclusive prefix sum of the block sizes
    DevTmp sz_mem, off_mem, scan_mem;
    HIPCHK(hipMalloc(&sz_mem.p, (size_t)nsub * sizeof(uint32_t)));
    HIPCHK(hipMalloc(&off_mem.p, (size_t)nsub * sizeof(uint32_t)));
    uint32_t *sz = static_cast<uint32_t *>(sz_mem.p), *blk_off = static_cast<uint32_t *>(off_mem.p);
    blk_size_kernel<<<dim3((unsigned)((nsub + 255) / 256)), dim3(256), 0, st>>>(d->sub_offsets, nsub, M, sz);
    LAUNCHCHK("blk_size_kernel");
    size_t tmp_bytes = 0;
    HIPCHK(rocprim::exclusive_scan(nullptr, tmp_bytes, sz, blk_off, 0u, (size_t)nsub,
                                   rocprim::plus<uint32_t>(), st));
    HIPCHK(hipMalloc(&scan_mem.p, tmp_bytes ? tmp_bytes : 16));
    HIPCHK(rocprim::exclusive_scan(scan_mem.p, tmp_bytes, sz, blk_off, 0u, (size_t)nsub,
                                   rocprim::plus<uint32_t>(), st));
    uint32_t last_off = 0, last_sz = 0;
    HIPCHK(hipMemcpyAsync(&last_off, blk_off + nsub - 1, 4, hipMemcpyDeviceToHost, st));
    HIPCHK(hipMemcpyAsync(&last_sz, sz + nsub - 1, 4, hipMemcpyDeviceToHost, st));
    HIPCHK(hipStreamSynchronize(st));
    const uint64_t total_blk = (uint64_t)last_off + last_sz;
    HIPCHK(hipMalloc(reinterpret_cast<void **>(&ix->blocks), (size_t)(total_blk ? total_blk : 1) * BLK_ALIGN));
    repack_kernel<<<dim3((unsigned)((nsub * 16 + 255) / 256)), dim3(256), 0, st>>>(
        d->sub_offsets, blk_off, nsub, M, d->codes, d->const_byte, ix->blocks);
    LAUNCHCHK("repack_kernel");
    HIPCHK(hipMalloc(reinterpret_cast<void **>(&ix->sub_info), (size_t)nsub * sizeof(uint4)));
    sub_info_kernel<<<dim3((unsigned)((nsub + 255) / 256)), dim3(256), 0, st>>>(d->sub_offsets, blk_off, nsub, ix->sub_info);
    LAUNCHCHK("sub_info_kernel");
    HIPCHK(hipStreamSynchronize(st));   // the temporaries are released on return
    return IVF_OK;
}

}  // namespace

extern "C" int ivf_load_index(const ivf_index_desc *d, void *hip_stream, ivf_index **out)
{
    int rc = check_trained(d);
    if (rc) return rc;
    if (!out) return fail(IVF_EINVAL, "out is NULL");
    if (!d->pq_codebook || !d->const_table || !d->sub_offsets || !d->codes || !d->const_byte || !d->ids)
        return fail(IVF_EINVAL, "pq_codebook or an encoded array (const_table, sub_offsets, codes, const_byte, ids) is NULL");
    if (d->N < 0 || d->N >= (1ll << 32)) return fail(IVF_EINVAL, "N=%lld out of range", (long long)d->N);
    if (!aligned16(d->codes)) return fail(IVF_EINVAL, "codes must be 16-byte aligned");
    ivf_index *ix = new (std::nothrow) ivf_index;
    if (!ix) return fail(IVF_ENOMEM, "host allocation failed");
    rc = load_impl(d, static_cast<hipStream_t>(hip_stream), ix);
    if (rc) {
        std::string keep = g_err;
        ivf_free_index(ix);
        g_err = keep;
        return rc;
    }
    *out = ix;
    return IVF_OK;
}

namespace {

struct SearchArgs {
    const float *queries;
    int64_t nq;
    int P, k, S;
    int32_t *out_ids;
    float *out_dists;
    int32_t *probe_id_out;
    float *probe_d_out;
    int64_t *kept_sub_out;
    int64_t *n_scanned_out;
    int64_t budget;          // candidate budget R, 0 = none
    uint8_t *visited_out;    // [nq][S] flags of the budget mode (may be NULL)
};

int check_search_args(const ivf_index *ix, const float *queries, int64_t nq, int nprobe, float prune_frac, int k,
                      const int32_t *out_ids, const float *out_dists)
{
    if (!ix) return fail(IVF_EINVAL, "index is NULL");
    if (nq < 0 || nq >= (1ll << 31)) return fail(IVF_EINVAL, "nq=%lld out of range", (long long)nq);
    if (nq == 0) return IVF_OK;
    if (!queries || !out_ids || !out_dists) return fail(IVF_EINVAL, "queries / out_ids / out_dists is NULL");
    if (!aligned16(queries)) return fail(IVF_EINVAL, "queries must be 16-byte aligned");
    if (nprobe < 1 || nprobe > ix->K || nprobe > 4096)
        return fail(IVF_EINVAL, "nprobe=%d must be in [1, min(K, 4096)]", nprobe);
    if (!(prune_frac > 0.f) || prune_frac > 1.f) return fail(IVF_EINVAL, "prune_frac must be in (0, 1]");
    if (k < 1 || k > IVF_MAX_K_RESULTS) return fail(IVF_EINVAL, "k=%d must be in [1, %d]", k, IVF_MAX_K_RESULTS);
    const int64_t PL = (int64_t)nprobe * ix->L;
    if (PL > IVF_MAX_SCORES) return fail(IVF_EINVAL, "nprobe*L=%lld exceeds %d", (long long)PL, IVF_MAX_SCORES);
    return IVF_OK;
}

// Dynamic LDS sizes of the stage kernels; raises the kernels' limits where they exceed the default window.
struct LdsPlan { size_t scan, merge, sp, ssp; };   // ssp: the fused selection + scoring launch of small batches

int plan_lds(const ivf_index *ix, int P, int k, const SearchPlan &pl, LdsPlan &l)
{
    const int64_t PL = (int64_t)P * ix->L;
    l.scan = (size_t)SCAN_WAVES * pool_capacity(k) * sizeof(uint64_t);   // dynamic part: the pools
    l.merge = ((size_t)pl.merge_n + pl.merge_pow2) * sizeof(uint64_t);
    l.sp = (size_t)(PL + 3 * P) * sizeof(uint32_t);
    if (l.sp < (size_t)ix->D * sizeof(float)) l.sp = (size_t)ix->D * sizeof(float);   // the table workgroups hold a query
    if (l.sp > 154 * 1024)   // one workgroup holds a query's scores in the 160 KB of LDS, beside 5 KB of static data
        return fail(IVF_EINVAL, "nprobe*L + 3*nprobe = %lld words exceed the LDS of one workgroup", (long long)(PL + 3 * P));
    if (l.sp > 48 * 1024) {
        const void *fn = PL > 16384 ? reinterpret_cast<const void *>(&score_prune_kernel<1024, 8>)
                         : PL > 4096 ? reinterpret_cast<const void *>(&score_prune_kernel<1024, 4>)
                                     : reinterpret_cast<const void *>(&score_prune_kernel<256, 4>);
        HIPCHK(hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)l.sp));
    }
    {   // the fused launch needs what either half needs (see launch_probe_select for the selection's share)
        const int64_t nb = (ix->K + BMW - 1) / BMW;
        const size_t sel = ((size_t)2 * P + 3 + (nb > 2 * PS_CAP ? nb : 2 * PS_CAP)) * sizeof(int);
        l.ssp = sel > l.sp ? sel : l.sp;
        if (P <= PS_P_MAX && nb <= PS_NB_MAX && PL > 4096 && l.ssp > 48 * 1024) {
            const void *fn = PL > 16384 ? reinterpret_cast<const void *>(&select_score_prune_kernel<8>)
                                        : reinterpret_cast<const void *>(&select_score_prune_kernel<4>);
            HIPCHK(hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)l.ssp));
        }
    }
    if (l.merge > 40 * 1024)
        HIPCHK(hipFuncSetAttribute(reinterpret_cast<const void *>(&merge_kernel<256>),
                                   hipFuncAttributeMaxDynamicSharedMemorySize, (int)l.merge));
    if (l.scan > 32 * 1024) {   // dynamic + static LDS above the default 64 KB window
        const void *fn = ix->M == 16 ? reinterpret_cast<const void *>(&scan_kernel<16>)
                                     : reinterpret_cast<const void *>(&scan_kernel<8>);
        HIPCHK(hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)l.scan));
    }
    return IVF_OK;
}

// The launch sequence of the query path over the batch, `pl.tile` queries per pass, on scratch the
// caller provides.  Allocates nothing (stage timing, which creates events, is the allocating
// entry points' option: `timed`).
int run_search(ivf_index *ix, const SearchArgs &a, const SearchPlan &pl, const LdsPlan &lds, const SearchWs &ws,
               bool timed, hipStream_t st)
{
    const int P = a.P, L = ix->L, M = ix->M, D = ix->D, S = a.S, k = a.k;
    const int64_t K = ix->K, PL = (int64_t)P * L;
    const int Dp = packed_dim(D);
    int rc;
    for (int64_t q0 = 0; q0 < a.nq; q0 += pl.tile) {
        const int64_t n = (a.nq - q0 < pl.tile) ? a.nq - q0 : pl.tile;
        const float *Q = a.queries + q0 * D;
        int32_t *pid = a.probe_id_out ? a.probe_id_out + q0 * P : ws.probe_id;
        float *pd = a.probe_d_out ? a.probe_d_out + q0 * P : ws.probe_d;

        auto mark = [&](int stage) -> int {
            if (!timed) return IVF_OK;
            hipEvent_t e;
            HIPCHK(hipEventCreate(&e));
            HIPCHK(hipEventRecord(e, st));
            ix->ev[stage].push_back(e);
            return IVF_OK;
        };
        if ((rc = mark(0))) return rc;
        if ((rc = pack_rows(Q, n, D, nullptr, ws.qpk, ws.qn, ws.qsi, st))) return rc;
        if ((rc = launch_coarse(ws.qpk, ws.qn, ws.qsi, n, ix->cpk, ix->cnorm, ix->csi, K, Dp, ws.dt, ws.bm, st))) return rc;
        if ((rc = mark(1))) return rc;
        // Where both are workgroups of 1024 threads with their keys in LDS, the selection runs inside the
        // scoring launch (one workgroup per query does both): one kernel boundary less, and the selection
        // of one query (LDS and ALU work) runs while the other workgroup of the CU waits for its gathers.
        const int nb = (int)((K + BMW - 1) / BMW);
        // (nprobe * L <= 4096 keeps the two launches: its scoring kernel runs 256 threads a workgroup, and
        // measured as one launch of 1024 it is slower: 1.33 against 0.44 + 0.85 ms on the 10^7-point workloads)
        const bool fused = P <= PS_P_MAX && nb <= PS_NB_MAX && PL > 4096;
        if (!fused && (rc = launch_probe_select(ws.dt, ws.bm, n, K, P, pid, pd, st))) return rc;
        if ((rc = mark(2))) return rc;

        int64_t *ks = a.kept_sub_out ? a.kept_sub_out + q0 * S : nullptr;
        int64_t *ns = a.n_scanned_out ? a.n_scanned_out + q0 : nullptr;
        const float *Qt = Q;                                   // what the lookup tables are built from
        if (ix->rot_t) {
            rotate_rows_kernel<<<dim3((unsigned)((n + ROT_ROWS - 1) / ROT_ROWS)), dim3(256), (size_t)ROT_ROWS * D * sizeof(float), st>>>(
                Q, n, D, ix->rot_t, ws.qrot);
            LAUNCHCHK("rotate_rows_kernel");
            Qt = ws.qrot;
        }
        // stages 2-3 (one workgroup per query) and stage 4 (one more workgroup per query) in one launch
#define IVF_SP_LAUNCH(BLK, MV)                                                                                     \
    score_prune_kernel<BLK, MV><<<dim3((unsigned)(2 * n)), dim3(BLK), lds.sp, st>>>(                                \
        ws.dt, dt_stride(K), K, pid, pd, P, L, ix->nbr, ix->cst, ix->alpha, S, ix->sub_info, ws.desc, ks, ns, n, Qt, \
        D, M, ix->codebook, ws.lut)
#define IVF_SSP_LAUNCH(MV)                                                                                          \
    select_score_prune_kernel<MV><<<dim3((unsigned)(2 * n)), dim3(1024), lds.ssp, st>>>(                             \
        ws.dt, dt_stride(K), ws.bm, K, nb, pid, pd, P, L, ix->nbr, ix->cst, ix->alpha, S, ix->sub_info, ws.desc, ks, ns, \
        n, Qt, D, M, ix->codebook, ws.lut)
        if (fused && PL > 16384) IVF_SSP_LAUNCH(8);
        else if (fused) IVF_SSP_LAUNCH(4);
        else if (PL > 16384) IVF_SP_LAUNCH(1024, 8);
        else if (PL > 4096) IVF_SP_LAUNCH(1024, 4);
        else IVF_SP_LAUNCH(256, 4);
#undef IVF_SP_LAUNCH
#undef IVF_SSP_LAUNCH
        LAUNCHCHK("score_prune_kernel");
        if (a.budget > 0) {
            const uint32_t R = a.budget > 0xFFFFFFFFll ? 0xFFFFFFFFu : (uint32_t)a.budget;
            budget_cut_kernel<256><<<dim3((unsigned)n), dim3(256), 0, st>>>(
                ws.desc, S, R, a.visited_out ? a.visited_out + q0 * S : nullptr, ns);
            LAUNCHCHK("budget_cut_kernel");
        }
        if ((rc = mark(3))) return rc;
        if ((rc = mark(4))) return rc;   // (the lookup tables are built inside the launch above)

        if (M == 16)
            scan_kernel<16><<<dim3((unsigned)(n * pl.nsplit)), dim3(SCAN_BLOCK), lds.scan, st>>>(
                ix->blocks, ix->const_table, ws.desc, S, ws.lut, k, pl.nsplit, ws.partial);
        else
            scan_kernel<8><<<dim3((unsigned)(n * pl.nsplit)), dim3(SCAN_BLOCK), lds.scan, st>>>(
                ix->blocks, ix->const_table, ws.desc, S, ws.lut, k, pl.nsplit, ws.partial);
        LAUNCHCHK("scan_kernel");
        if ((rc = mark(5))) return rc;

        merge_kernel<256><<<dim3((unsigned)n), dim3(256), lds.merge, st>>>(
            ws.partial, ix->ids, pl.merge_n, pl.merge_pow2, k, a.out_ids + q0 * k, a.out_dists + q0 * k);
        LAUNCHCHK("merge_kernel");
        if ((rc = mark(6))) return rc;
        if (timed) ix->launches++;
    }
    return IVF_OK;
}

// Scratch for callers that must not allocate: one array per GPU, part of the loaded code object,
// so it exists from the moment the library is loaded until the process ends.  Host code never uses
// the array's name as an address; it asks the runtime for the array's device address once per
// device and keeps that.
static __device__ __align__(256) unsigned char scratch[IVF_NOALLOC_SCRATCH_BYTES];

constexpr int MAX_DEVICES = 64;
std::mutex g_scratch_mu;
unsigned char *g_scratch_ptr[MAX_DEVICES] = {};

// Device address of this GPU's copy of `scratch` (the current device).
int scratch_of_current_device(unsigned char **out)
{
    int dev = -1;
    HIPCHK(hipGetDevice(&dev));
    if (dev < 0 || dev >= MAX_DEVICES) return fail(IVF_EINVAL, "device ordinal %d out of range", dev);
    std::lock_guard<std::mutex> lock(g_scratch_mu);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        HIPCHK(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        if (!p) return fail(IVF_EHIP, "hipGetSymbolAddress returned a null address");
        g_scratch_ptr[dev] = static_cast<unsigned char *>(p);
    }
    *out = g_scratch_ptr[dev];
    return IVF_OK;
}

// The query path on the handle's own growable scratch (allocates when a call needs more than any before).
int search_alloc(ivf_index *ix, const float *queries, int64_t nq, int nprobe, float prune_frac, int k,
                 int32_t *out_ids, float *out_dists, int32_t *probe_id_out, float *probe_d_out,
                 int64_t *kept_sub_out, int64_t *n_scanned_out, int64_t budget, uint8_t *visited_out,
                 void *hip_stream)
{
    int rc = check_search_args(ix, queries, nq, nprobe, prune_frac, k, out_ids, out_dists);
    if (rc || nq == 0) return rc;
    const int64_t K = ix->K;
    const int S = (int)ivf_num_kept(nprobe, ix->L, prune_frac);
    hipStream_t st = static_cast<hipStream_t>(hip_stream);

    // queries per pass: bounded by the distance tile
    int64_t tile = ix->scratch_limit / (K * (int64_t)sizeof(float));
    if (tile < 1) tile = 1;
    if (tile >= nq) tile = nq;
    else if (tile >= 256) tile -= tile % 256;   // whole blocks of the padded row count
    else if (tile >= GT) tile -= tile % GT;

    const SearchPlan pl = plan_search(K, ix->D, ix->M, nprobe, S, k, tile, ix->rot_t != nullptr);
    Buf *bufs[WS_COUNT] = {&ix->dt, &ix->bm, &ix->qn, &ix->qsi, &ix->qpk, &ix->probe_id, &ix->probe_d,
                           &ix->desc, &ix->lut, &ix->partial, &ix->qrot};
    for (int i = 0; i < WS_COUNT; ++i)
        if ((rc = ensure(*bufs[i], pl.bytes[i]))) return rc;
    SearchWs ws;
    ws.dt = static_cast<float *>(ix->dt.p);
    ws.bm = static_cast<float *>(ix->bm.p);
    ws.qn = static_cast<float *>(ix->qn.p);
    ws.qsi = static_cast<float *>(ix->qsi.p);
    ws.qpk = static_cast<_Float16 *>(ix->qpk.p);
    ws.probe_id = static_cast<int32_t *>(ix->probe_id.p);
    ws.probe_d = static_cast<float *>(ix->probe_d.p);
    ws.desc = static_cast<SubDesc *>(ix->desc.p);
    ws.lut = static_cast<float *>(ix->lut.p);
    ws.partial = static_cast<uint64_t *>(ix->partial.p);
    ws.qrot = static_cast<float *>(ix->qrot.p);
    LdsPlan lds;
    if ((rc = plan_lds(ix, nprobe, k, pl, lds))) return rc;
    const SearchArgs a = {queries, nq, nprobe, k, S, out_ids, out_dists, probe_id_out, probe_d_out, kept_sub_out,
                          n_scanned_out, budget, visited_out};
    return run_search(ix, a, pl, lds, ws, ix->profile, st);
}

}  // namespace

extern "C" int ivf_search_stages(ivf_index *ix, const float *queries, int64_t nq, int nprobe,
                                 float prune_frac, int k, int32_t *out_ids, float *out_dists,
                                 int32_t *probe_id_out, float *probe_d_out, int64_t *kept_sub_out,
                                 int64_t *n_scanned_out, void *hip_stream)
{
    return search_alloc(ix, queries, nq, nprobe, prune_frac, k, out_ids, out_dists, probe_id_out, probe_d_out,
                        kept_sub_out, n_scanned_out, 0, nullptr, hip_stream);
}

extern "C" int ivf_search_budget(ivf_index *ix, const float *queries, int64_t nq, int nprobe, float prune_frac,
                                 int64_t max_candidates, int k, int32_t *out_ids, float *out_dists,
                                 int64_t *kept_sub_out, uint8_t *visited_out, int64_t *n_scanned_out,
                                 void *hip_stream)
{
    if (max_candidates < 1) return fail(IVF_EINVAL, "max_candidates=%lld must be positive", (long long)max_candidates);
    return search_alloc(ix, queries, nq, nprobe, prune_frac, k, out_ids, out_dists, nullptr, nullptr,
                        kept_sub_out, n_scanned_out, max_candidates, visited_out, hip_stream);
}

extern "C" int ivf_search_noalloc(ivf_index *ix, const float *queries, int64_t nq, int nprobe, float prune_frac,
                                  int k, int32_t *out_ids, float *out_dists, void *hip_stream)
{
    int rc = check_search_args(ix, queries, nq, nprobe, prune_frac, k, out_ids, out_dists);
    if (rc || nq == 0) return rc;
    const int S = (int)ivf_num_kept(nprobe, ix->L, prune_frac);
    // the whole batch in one pass: the scratch is carved out of the static array, 256-byte aligned pieces
    const SearchPlan pl = plan_search(ix->K, ix->D, ix->M, nprobe, S, k, nq, ix->rot_t != nullptr);
    size_t off[WS_COUNT], total = 0;
    for (int i = 0; i < WS_COUNT; ++i) {
        off[i] = total;
        total += (pl.bytes[i] + 255) / 256 * 256;
    }
    if (total > (size_t)IVF_NOALLOC_SCRATCH_BYTES)
        return fail(IVF_EINVAL, "ivf_search_noalloc: this batch needs %zu bytes of scratch, the static array holds %zu "
                    "(nq=%lld, K=%lld); use fewer queries per call or ivf_search",
                    total, (size_t)IVF_NOALLOC_SCRATCH_BYTES, (long long)nq, (long long)ix->K);
    unsigned char *base = nullptr;
    if ((rc = scratch_of_current_device(&base))) return rc;
    SearchWs ws;
    ws.dt = reinterpret_cast<float *>(base + off[WS_DT]);
    ws.bm = reinterpret_cast<float *>(base + off[WS_BM]);
    ws.qn = reinterpret_cast<float *>(base + off[WS_QN]);
    ws.qsi = reinterpret_cast<float *>(base + off[WS_QSI]);
    ws.qpk = reinterpret_cast<_Float16 *>(base + off[WS_QPK]);
    ws.probe_id = reinterpret_cast<int32_t *>(base + off[WS_PID]);
    ws.probe_d = reinterpret_cast<float *>(base + off[WS_PD]);
    ws.desc = reinterpret_cast<SubDesc *>(base + off[WS_DESC]);
    ws.lut = reinterpret_cast<float *>(base + off[WS_LUT]);
    ws.partial = reinterpret_cast<uint64_t *>(base + off[WS_PARTIAL]);
    ws.qrot = reinterpret_cast<float *>(base + off[WS_QROT]);
    LdsPlan lds;
    if ((rc = plan_lds(ix, nprobe, k, pl, lds))) return rc;
    const SearchArgs a = {queries, nq, nprobe, k, S, out_ids, out_dists, nullptr, nullptr, nullptr, nullptr, 0, nullptr};
    return run_search(ix, a, pl, lds, ws, false, static_cast<hipStream_t>(hip_stream));
}

extern "C" int ivf_profile_enable(ivf_index *ix, int on)
{
    if (!ix) return fail(IVF_EINVAL, "index is NULL");
    ix->profile = on != 0;
    return IVF_OK;
}

extern "C" int ivf_profile_read(ivf_index *ix, double *stage_ms, int64_t *launches)
{
    if (!ix || !stage_ms || !launches) return fail(IVF_EINVAL, "NULL argument");
    HIPCHK(hipDeviceSynchronize());
    for (int s = 0; s < IVF_N_STAGES; ++s) {
        double tot = 0.0;
        for (size_t i = 0; i < ix->ev[s].size() && i < ix->ev[s + 1].size(); ++i) {
            float ms = 0.f;
            HIPCHK(hipEventElapsedTime(&ms, ix->ev[s][i], ix->ev[s + 1][i]));
            tot += ms;
        }
        stage_ms[s] = tot;
    }
    *launches = ix->launches;
    for (int s = 0; s <= IVF_N_STAGES; ++s) {
        for (hipEvent_t e : ix->ev[s]) (void)hipEventDestroy(e);
        ix->ev[s].clear();
    }
    ix->launches = 0;
    return IVF_OK;
}

extern "C" int ivf_search(ivf_index *ix, const float *queries, int64_t nq, int nprobe, float prune_frac,
                          int k, int32_t *out_ids, float *out_dists, void *hip_stream)
{
    return ivf_search_stages(ix, queries, nq, nprobe, prune_frac, k, out_ids, out_dists, nullptr,
                             nullptr, nullptr, nullptr, hip_stream);
}

namespace {

std::atomic<int64_t> g_assign_short{0}, g_assign_exact{0};

// Nearest-centroid assignment (P = 1) with buffers that live across calls: the packed centroid
// table and the per-chunk query scratch.  No distance tile: the minimum is fused into the GEMM.
//
// Two passes: the hi halves of the operands alone (a third of the MFMA work) give every row a short
// list of centroids that may be its nearest, with a proven error bound (coarse_shortlist_kernel), and
// the exact distances of the listed pairs decide (rerank_kernel).  A chunk whose list overflows (rows
// with very many centroids at nearly the same distance) is redone by the exact kernel.
struct ArgminCtx {
    int64_t K = 0, chunk = 0;
    int D = 0, Dp = 0;
    float *cn = nullptr, *csi = nullptr, *xn = nullptr, *xsi = nullptr;
    _Float16 *cpk = nullptr, *xpk = nullptr, *chk = nullptr, *xhk = nullptr;   // hi/lo tables, hi-only tables
    unsigned long long *best = nullptr, *cand_count = nullptr;
    uint32_t *U = nullptr;
    int2 *cand = nullptr;
    unsigned long long seg_cap = 0;
    const float *centroids = nullptr;          // the caller's table, as of the last set_centroids
    bool shortlist = true;
    int64_t chunks_short = 0, chunks_exact = 0;   // how the chunks of all run() calls were decided
    ArgminCtx() = default;
    ArgminCtx(const ArgminCtx &) = delete;
    ArgminCtx &operator=(const ArgminCtx &) = delete;
    ~ArgminCtx()
    {
        void *owned[] = {cn, csi, xn, xsi, cpk, xpk, chk, xhk, best, cand_count, U, cand};
        for (void *p : owned)
            if (p) (void)hipFree(p);
    }
    int init(int64_t K_, int D_, int64_t max_rows)
    {
        K = K_; D = D_; Dp = packed_dim(D);
        // rows per launch: at most 2^20, and few enough that the grid (one workgroup of 256 threads per
        // tile of 128 rows x 128 centroids) stays below the 2^32 threads a launch may have
        const int64_t tiles_c = (K + GT - 1) / GT;
        int64_t max_tq = ((1ll << 24) - 1) / tiles_c / N_XCD * N_XCD;
        if (max_tq < N_XCD) return fail(IVF_EINVAL, "K=%lld: too many centroid tiles for one launch", (long long)K);
        chunk = max_tq * GT < (1ll << 20) ? max_tq * GT : (1ll << 20);
        if (max_rows < chunk) chunk = max_rows > 0 ? max_rows : 1;
        HIPCHK(hipMalloc(reinterpret_cast<void **>(&cn), (size_t)K * sizeof(float)));
        HIPCHK(hipMalloc(reinterpret_cast<void **>(&cpk), (size_t)packed_rows(K) * Dp * 2 * sizeof(_Float16)));
        HIPCHK(hipMalloc(reinterpret_cast<void **>(&csi), 2 * sizeof(float)));
        HIPCHK(hipMalloc(reinterpret_cast<void **>(&xn), (size_t)chunk * sizeof(float)));
        HIPCHK(hipMalloc(reinterpret_cast<void **>(&xsi), (size_t)chunk * sizeof(float)));
        HIPCHK(hipMalloc(reinterpret_cast<void **>(&xpk), (size_t)packed_rows(chunk) * Dp * 2 * sizeof(_Float16)));
        HIPCHK(hipMalloc(reinterpret_cast<void **>(&best), (size_t)chunk * sizeof(unsigned long long)));
        const char *off = getenv("IVF_GP_EXACT_ASSIGN");   // (for measurements: the one-pass exact kernel only)
        shortlist = !(off && off[0] == '1');
        if (shortlist) {
            // room for 32 listed centroids per row on average, at least 2^16 pairs per segment
            seg_cap = (unsigned long long)(32 * chunk + SHORTLIST_SEGS - 1) / SHORTLIST_SEGS;
            if (seg_cap < (1ull << 16)) seg_cap = 1ull << 16;
            HIPCHK(hipMalloc(reinterpret_cast<void **>(&chk), (size_t)packed_rows(K) * Dp * sizeof(_Float16)));
            HIPCHK(hipMalloc(reinterpret_cast<void **>(&xhk), (size_t)packed_rows(chunk) * Dp * sizeof(_Float16)));
            HIPCHK(hipMalloc(reinterpret_cast<void **>(&U), (size_t)(chunk + 2) * sizeof(uint32_t)));   // filled in 64-bit words
            HIPCHK(hipMalloc(reinterpret_cast<void **>(&cand), (size_t)seg_cap * SHORTLIST_SEGS * sizeof(int2)));
            HIPCHK(hipMalloc(reinterpret_cast<void **>(&cand_count), (size_t)SHORTLIST_SEGS * 16 * sizeof(unsigned long long)));
        }
        return IVF_OK;
    }
    int set_centroids(const float *centroids_, hipStream_t st)
    {
        centroids = centroids_;
        int rc = pack_rows(centroids, K, D, reinterpret_cast<uint32_t *>(csi + 1), cpk, cn, csi, st);
        if (rc || !shortlist) return rc;
        const int64_t chunks16 = K * (Dp / 8);
        pack_hi_kernel<<<dim3((unsigned)((chunks16 + 255) / 256)), dim3(256), 0, st>>>(cpk, K, Dp, chk);
        LAUNCHCHK("pack_hi_kernel");
        return IVF_OK;
    }
    // the exact one-pass kernel on the packed chunk
    int run_exact(int64_t m, hipStream_t st)
    {
        const int tiles_q = (int)((m + GT - 1) / GT);
        const int64_t grid = (int64_t)((tiles_q + N_XCD - 1) / N_XCD) * N_XCD * ((K + GT - 1) / GT);
        if (grid >= (1ll << 24)) return fail(IVF_EINVAL, "coarse tile grid too large");
        fill_u64_kernel<<<dim3((unsigned)((m + 255) / 256)), dim3(256), 0, st>>>(best, m, ~0ull);
        LAUNCHCHK("fill_u64_kernel");
        coarse_argmin_kernel<<<dim3((unsigned)grid), dim3(256), 0, st>>>(xpk, xn, xsi, m, cpk, cn, csi, K, Dp, best, tiles_q);
        LAUNCHCHK("coarse_argmin_kernel");
        ++chunks_exact; ++g_assign_exact;
        return IVF_OK;
    }
    // shortlist + exact decision; *overflow = the list did not hold every candidate (best[] is then incomplete)
    int run_shortlist(const float *x, int64_t m, bool *overflow, hipStream_t st)
    {
        const int tiles_q = (int)((m + GT - 1) / GT);
        const int64_t grid = (int64_t)((tiles_q + N_XCD - 1) / N_XCD) * N_XCD * ((K + GT - 1) / GT);
        if (grid >= (1ll << 24)) return fail(IVF_EINVAL, "coarse tile grid too large");
        const int64_t chunks16 = m * (Dp / 8);
        pack_hi_kernel<<<dim3((unsigned)((chunks16 + 255) / 256)), dim3(256), 0, st>>>(xpk, m, Dp, xhk);
        LAUNCHCHK("pack_hi_kernel");
        fill_u64_kernel<<<dim3((unsigned)((m + 255) / 256)), dim3(256), 0, st>>>(best, m, ~0ull);
        LAUNCHCHK("fill_u64_kernel");
        // U: 32-bit words, two per 64-bit fill; the counters likewise
        fill_u64_kernel<<<dim3((unsigned)(((m + 1) / 2 + 255) / 256)), dim3(256), 0, st>>>(reinterpret_cast<unsigned long long *>(U), (m + 1) / 2, ~0ull);
        LAUNCHCHK("fill_u64_kernel");
        fill_u64_kernel<<<dim3((SHORTLIST_SEGS * 16 + 255) / 256), dim3(256), 0, st>>>(cand_count, SHORTLIST_SEGS * 16, 0ull);
        LAUNCHCHK("fill_u64_kernel");
        if (Dp == 96 || Dp == 128) {   // query tile in registers, centroid tiles swept
            const int per_wg = 64;
            const int64_t tiles_c = (K + GT - 1) / GT;
            const int64_t g2 = (int64_t)((tiles_q + N_XCD - 1) / N_XCD) * N_XCD * ((tiles_c + per_wg - 1) / per_wg);
            if (Dp == 96)
                coarse_shortlist_sweep_kernel<3><<<dim3((unsigned)g2), dim3(256), 0, st>>>(xhk, xn, xsi, m, chk, cn, csi, K, D, U, cand, cand_count,
                                                                                         seg_cap, tiles_q, (int)tiles_c, per_wg);
            else
                coarse_shortlist_sweep_kernel<4><<<dim3((unsigned)g2), dim3(256), 0, st>>>(xhk, xn, xsi, m, chk, cn, csi, K, D, U, cand, cand_count,
                                                                                         seg_cap, tiles_q, (int)tiles_c, per_wg);
            LAUNCHCHK("coarse_shortlist_sweep_kernel");
        } else {
            coarse_shortlist_kernel<<<dim3((unsigned)grid), dim3(256), 0, st>>>(xhk, xn, xsi, m, chk, cn, csi, K, Dp / 2, D, U, cand,
                                                                                cand_count, seg_cap, tiles_q);
            LAUNCHCHK("coarse_shortlist_kernel");
        }
        unsigned long long counts[SHORTLIST_SEGS * 16];
        HIPCHK(hipMemcpyAsync(counts, cand_count, sizeof(counts), hipMemcpyDeviceToHost, st));
        HIPCHK(hipStreamSynchronize(st));
        unsigned long long longest = 0;
        for (int sgm = 0; sgm < SHORTLIST_SEGS; ++sgm) longest = counts[sgm * 16] > longest ? counts[sgm * 16] : longest;
        *overflow = longest > seg_cap || longest == 0;
        if (*overflow) return IVF_OK;
        rerank_kernel<<<dim3((unsigned)((longest + 3) / 4), SHORTLIST_SEGS), dim3(256), 0, st>>>(x, centroids, D, cand, cand_count, seg_cap, best);
        LAUNCHCHK("rerank_kernel");
        ++chunks_short; ++g_assign_short;
        return IVF_OK;
    }
    // out_id[i] = nearest centroid of x[i] by (distance, id), out_d[i] (may be NULL) its squared distance
    int run(const float *x, int64_t n, int32_t *out_id, float *out_d, hipStream_t st)
    {
        int rc;
        for (int64_t q0 = 0; q0 < n; q0 += chunk) {
            const int64_t m = (n - q0 < chunk) ? n - q0 : chunk;
            if ((rc = pack_rows(x + q0 * D, m, D, nullptr, xpk, xn, xsi, st))) return rc;
            bool overflow = true;
            if (shortlist && (rc = run_shortlist(x + q0 * D, m, &overflow, st))) return rc;
            if (overflow && (rc = run_exact(m, st))) return rc;
            argmin_unpack_kernel<<<dim3((unsigned)((m + 255) / 256)), dim3(256), 0, st>>>(best, m, out_id + q0, out_d ? out_d + q0 : nullptr);
            LAUNCHCHK("argmin_unpack_kernel");
        }
        return IVF_OK;
    }
};

int check_coarse_args(const float *centroids, int64_t K, int D, const float *x, int64_t nq)
{
    if (!centroids || !x) return fail(IVF_EINVAL, "NULL argument");
    if (D < 4 || D % 4 || D > IVF_MAX_D) return fail(IVF_EINVAL, "D=%d must be a multiple of 4 in [4, %d]", D, IVF_MAX_D);
    if (K < 1 || K >= (1ll << 31)) return fail(IVF_EINVAL, "K=%lld out of range", (long long)K);
    if (nq < 0 || nq >= (1ll << 31)) return fail(IVF_EINVAL, "row count out of range");
    if (!aligned16(centroids) || !aligned16(x)) return fail(IVF_EINVAL, "centroids and x must be 16-byte aligned");
    return IVF_OK;
}

// The P nearest centroids of every row of x through the distance tile (P > 1), on scratch of its own.
int coarse_topk_tiled(const float *centroids, int64_t K, int D, const float *x, int64_t nq, int P,
                      int32_t *out_id, float *out_d, hipStream_t st)
{
    int64_t tile = (4ll << 30) / (K * (int64_t)sizeof(float));
    if (tile < 1) tile = 1;
    if (tile >= nq) tile = nq;
    else if (tile >= 256) tile -= tile % 256;   // whole blocks of the padded row count
    else if (tile >= GT) tile -= tile % GT;
    const int64_t nb = (K + BMW - 1) / BMW;
    const int Dp = packed_dim(D);
    DevTmp cn, csi, cpk, xn, xsi, xpk, Dt, bm;
    HIPCHK(hipMalloc(&cn.p, (size_t)K * sizeof(float)));
    HIPCHK(hipMalloc(&cpk.p, (size_t)packed_rows(K) * Dp * 2 * sizeof(_Float16)));
    HIPCHK(hipMalloc(&csi.p, 2 * sizeof(float)));
    const size_t tile_pad = (size_t)packed_rows(tile);   // the GEMM may write whole tiles of rows
    HIPCHK(hipMalloc(&xn.p, tile_pad * sizeof(float)));
    HIPCHK(hipMalloc(&xsi.p, tile_pad * sizeof(float)));
    HIPCHK(hipMalloc(&xpk.p, tile_pad * Dp * 2 * sizeof(_Float16)));
    HIPCHK(hipMalloc(&Dt.p, tile_pad * dt_stride(K) * sizeof(float)));
    HIPCHK(hipMalloc(&bm.p, tile_pad * nb * sizeof(float)));
    float *csi_f = static_cast<float *>(csi.p);
    int rc = pack_rows(centroids, K, D, reinterpret_cast<uint32_t *>(csi_f + 1), static_cast<_Float16 *>(cpk.p),
                       static_cast<float *>(cn.p), csi_f, st);
    for (int64_t q0 = 0; q0 < nq && !rc; q0 += tile) {
        const int64_t n = (nq - q0 < tile) ? nq - q0 : tile;
        if ((rc = pack_rows(x + q0 * D, n, D, nullptr, static_cast<_Float16 *>(xpk.p), static_cast<float *>(xn.p),
                            static_cast<float *>(xsi.p), st))) break;
        if ((rc = launch_coarse(static_cast<_Float16 *>(xpk.p), static_cast<float *>(xn.p), static_cast<float *>(xsi.p), n,
                                static_cast<_Float16 *>(cpk.p), static_cast<float *>(cn.p), csi_f, K, Dp,
                                static_cast<float *>(Dt.p), static_cast<float *>(bm.p), st))) break;
        rc = launch_probe_select(static_cast<float *>(Dt.p), static_cast<float *>(bm.p), n, K, P, out_id + q0 * P,
                                 out_d + q0 * P, st);
    }
    std::string keep = g_err;
    (void)hipStreamSynchronize(st);   // the temporaries are released on return
    g_err = keep;
    return rc;
}

}  // namespace

extern "C" void ivf_assign_stats(int64_t *out)
{
    out[0] = g_assign_short.load();
    out[1] = g_assign_exact.load();
}

extern "C" int ivf_coarse_topk(const float *centroids, int64_t K, int D, const float *x, int64_t nq, int P,
                               int32_t *out_id, float *out_d, void *hip_stream)
{
    int rc = check_coarse_args(centroids, K, D, x, nq);
    if (rc) return rc;
    if (!out_id || !out_d) return fail(IVF_EINVAL, "NULL argument");
    if (P < 1 || P > K || P > 4096) return fail(IVF_EINVAL, "need 1 <= P <= min(K, 4096)");
    if (nq == 0) return IVF_OK;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    if (P > 1) return coarse_topk_tiled(centroids, K, D, x, nq, P, out_id, out_d, st);
    ArgminCtx ctx;   // fused per-row minimum, no distance tile
    if ((rc = ctx.init(K, D, nq))) return rc;
    if (!(rc = ctx.set_centroids(centroids, st))) rc = ctx.run(x, nq, out_id, out_d, st);
    std::string keep = g_err;
    (void)hipStreamSynchronize(st);
    g_err = keep;
    return rc;
}

extern "C" int ivf_encode(const ivf_index_desc *t, const float *x, int64_t n, const int32_t *region_in,
                          int32_t *out_region, int32_t *out_sub, uint8_t *out_codes,
                          uint8_t *out_const_byte, float *out_const_t, float *out_residual,
                          void *hip_stream)
{
    int rc = check_trained(t);
    if (rc) return rc;
    if (!x || !out_region || !out_sub) return fail(IVF_EINVAL, "NULL argument");
    if (t->pq_codebook && !out_codes) return fail(IVF_EINVAL, "out_codes is NULL");
    if (t->pq_codebook && !aligned16(t->pq_codebook)) return fail(IVF_EINVAL, "pq_codebook must be 16-byte aligned");
    if (t->pq_codebook && t->const_table && !out_const_byte) return fail(IVF_EINVAL, "out_const_byte is NULL");
    if (!aligned16(x)) return fail(IVF_EINVAL, "x must be 16-byte aligned");
    if (n < 0 || n >= (1ll << 31)) return fail(IVF_EINVAL, "n out of range");
    if (n == 0) return IVF_OK;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    if (region_in) {
        if (region_in != out_region)
            HIPCHK(hipMemcpyAsync(out_region, region_in, (size_t)n * sizeof(int32_t), hipMemcpyDeviceToDevice, st));
    } else {
        float *d1 = nullptr;
        HIPCHK(hipMalloc(reinterpret_cast<void **>(&d1), (size_t)n * sizeof(float)));
        rc = ivf_coarse_topk(t->centroids, t->K, t->D, x, n, 1, out_region, d1, hip_stream);
        std::string keep = g_err;
        (void)hipFree(d1);
        g_err = keep;
        if (rc) return rc;
    }
    // PQ codes by the thread-per-point kernel when the codebook fits LDS and D / M is one of the
    // compiled block widths; else by the wavefront-per-point kernel, which does everything.
    const int ds = t->D / t->M;
    const size_t cb_bytes = (size_t)256 * t->D * sizeof(float);
    const bool fast = t->pq_codebook && cb_bytes <= 140 * 1024 &&
                      (ds == 4 || ds == 6 || ds == 8 || ds == 12 || ds == 16);
    if (t->rotation && t->pq_codebook && !fast)
        return fail(IVF_EINVAL, "a rotation in front of the PQ needs D/M in {4, 6, 8, 12, 16} and a codebook that fits LDS");
    if (!fast) {
        encode_kernel<<<dim3((unsigned)n), dim3(64), (size_t)4 * t->D * sizeof(float), st>>>(
            x, n, t->D, t->M, t->L, out_region, t->centroids, t->nbr, t->alpha, t->cs_dist2, t->pq_codebook,
            t->const_table, out_sub, out_codes, out_const_byte, out_const_t, out_residual, nullptr);
        LAUNCHCHK("encode_kernel");
        HIPCHK(hipStreamSynchronize(st));
        return IVF_OK;
    }
    const int64_t chunk = n < (1ll << 20) ? n : (1ll << 20);
    const int D = t->D;
    DevTmp e, mu, erot, rt;
    auto body = [&]() -> int {
        if (!out_residual) HIPCHK(hipMalloc(&e.p, (size_t)chunk * D * sizeof(float)));
        HIPCHK(hipMalloc(&mu.p, (size_t)chunk * D * sizeof(float)));
        if (t->rotation) {   // the PQ sees R (x - mu), the per-point constant is taken with R mu
            HIPCHK(hipMalloc(&erot.p, (size_t)chunk * D * sizeof(float)));
            HIPCHK(hipMalloc(&rt.p, (size_t)D * D * sizeof(float)));
            transpose_square_kernel<<<dim3((unsigned)((D * D + 255) / 256)), dim3(256), 0, st>>>(t->rotation, D, static_cast<float *>(rt.p));
            LAUNCHCHK("transpose_square_kernel");
        }
        const void *fn = ds == 4 ? (const void *)&pq_encode_kernel<4> : ds == 6 ? (const void *)&pq_encode_kernel<6>
                       : ds == 8 ? (const void *)&pq_encode_kernel<8> : ds == 12 ? (const void *)&pq_encode_kernel<12>
                                                                                 : (const void *)&pq_encode_kernel<16>;
        HIPCHK(hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)cb_bytes));
        float *muc = static_cast<float *>(mu.p);
        for (int64_t i0 = 0; i0 < n; i0 += chunk) {
            const int64_t m = n - i0 < chunk ? n - i0 : chunk;
            float *ec = out_residual ? out_residual + i0 * D : static_cast<float *>(e.p);
            encode_kernel<<<dim3((unsigned)m), dim3(64), (size_t)4 * D * sizeof(float), st>>>(
                x + i0 * D, m, D, t->M, t->L, out_region + i0, t->centroids, t->nbr, t->alpha, t->cs_dist2,
                nullptr, nullptr, out_sub + i0, nullptr, nullptr, nullptr, ec, muc);
            LAUNCHCHK("encode_kernel");
            const float *pe = ec;
            if (t->rotation) {
                const unsigned rg = (unsigned)((m + ROT_ROWS - 1) / ROT_ROWS);
                const size_t rl = (size_t)ROT_ROWS * D * sizeof(float);
                rotate_rows_kernel<<<dim3(rg), dim3(256), rl, st>>>(ec, m, D, static_cast<float *>(rt.p), static_cast<float *>(erot.p));
                LAUNCHCHK("rotate_rows_kernel");
                rotate_rows_kernel<<<dim3(rg), dim3(256), rl, st>>>(muc, m, D, static_cast<float *>(rt.p), muc);
                LAUNCHCHK("rotate_rows_kernel");
                pe = static_cast<float *>(erot.p);
            }
            int64_t grid = (m + 1023) / 1024;
            if (grid > 512) grid = 512;
            uint8_t *oc = out_codes + i0 * t->M;
            uint8_t *ob = out_const_byte ? out_const_byte + i0 : nullptr;
            float *ot = out_const_t ? out_const_t + i0 : nullptr;
#define IVF_PQ_LAUNCH(DSV)                                                                               \
    pq_encode_kernel<DSV><<<dim3((unsigned)grid), dim3(1024), cb_bytes, st>>>(pe, muc, m, t->M, t->pq_codebook, \
                                                                               t->const_table, oc, ob, ot)
            if (ds == 4) IVF_PQ_LAUNCH(4);
            else if (ds == 6) IVF_PQ_LAUNCH(6);
            else if (ds == 8) IVF_PQ_LAUNCH(8);
            else if (ds == 12) IVF_PQ_LAUNCH(12);
            else IVF_PQ_LAUNCH(16);
#undef IVF_PQ_LAUNCH
            LAUNCHCHK("pq_encode_kernel");
        }
        HIPCHK(hipStreamSynchronize(st));
        return IVF_OK;
    };
    rc = body();
    {
        std::string keep = g_err;
        (void)hipStreamSynchronize(st);   // the temporaries are released on return
        g_err = keep;
    }
    return rc;
}

extern "C" int ivf_rotate(const float *x, int64_t n, int D, const float *rotation, float *out, void *hip_stream)
{
    if (!x || !rotation || !out) return fail(IVF_EINVAL, "NULL argument");
    if (D < 1 || D > IVF_MAX_D || n < 0 || n >= (1ll << 31)) return fail(IVF_EINVAL, "bad sizes");
    if (n == 0) return IVF_OK;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    DevTmp rt;
    HIPCHK(hipMalloc(&rt.p, (size_t)D * D * sizeof(float)));
    transpose_square_kernel<<<dim3((unsigned)((D * D + 255) / 256)), dim3(256), 0, st>>>(rotation, D, static_cast<float *>(rt.p));
    int rc = IVF_OK;
    hipError_t e1 = hipGetLastError();
    if (e1 != hipSuccess) rc = fail(IVF_EHIP, "launch transpose_square_kernel: %s", hipGetErrorString(e1));
    if (!rc) {
        rotate_rows_kernel<<<dim3((unsigned)((n + ROT_ROWS - 1) / ROT_ROWS)), dim3(256), (size_t)ROT_ROWS * D * sizeof(float), st>>>(
            x, n, D, static_cast<float *>(rt.p), out);
        e1 = hipGetLastError();
        if (e1 != hipSuccess) rc = fail(IVF_EHIP, "launch rotate_rows_kernel: %s", hipGetErrorString(e1));
    }
    std::string keep = g_err;
    (void)hipStreamSynchronize(st);
    g_err = keep;
    return rc;
}

extern "C" int ivf_copy_bytes(void *dst, const void *src, int64_t nbytes, void *hip_stream)
{
    if (!dst || !src || nbytes < 0 || nbytes % 16 || !aligned16(dst) || !aligned16(src))
        return fail(IVF_EINVAL, "ivf_copy_bytes needs 16-byte aligned pointers and a multiple of 16 bytes");
    if (nbytes == 0) return IVF_OK;
    const int64_t n16 = nbytes / 16;
    int64_t grid = (n16 + 255) / 256;
    if (grid > 256 * 32) grid = 256 * 32;
    copy_bytes_kernel<<<dim3((unsigned)grid), dim3(256), 0, static_cast<hipStream_t>(hip_stream)>>>(
        static_cast<const uint4 *>(src), static_cast<uint4 *>(dst), n16);
    LAUNCHCHK("copy_bytes_kernel");
    return IVF_OK;
}

#include "train_api.hpp"
