// Host side of the index-time training entry points (included by ivf_gp.hip, after its helpers).
#pragma once

namespace {

inline unsigned grid_for(int64_t n, int block = 256) { return (unsigned)((n + block - 1) / block); }

// Stable sort of n (key, value) pairs by the low `bits` bits of the key, ascending: one
// least-significant-digit pass per 8 bits.  vals_in == NULL: the values are the positions 0..n-1.
// The sorted pairs end up in *keys_sorted / *vals_sorted, which point into the caller's two pairs
// of buffers (a: first, b: second; keys_in may be the a buffer).  hist: 256 * nblocks words,
// scan_tmp: temporary of rocprim's scan (scan_bytes).
struct RadixBufs {
    DevTmp ka, kb, va, vb, hist, base, scan;
    size_t scan_bytes = 0;
    int64_t nblocks = 0, cap = 0;
    int init(int64_t n)
    {
        cap = n;
        nblocks = (n + RS_TILE - 1) / RS_TILE;
        if (nblocks < 1) nblocks = 1;
        const size_t nb = (size_t)(n > 0 ? n : 1) * sizeof(uint32_t);
        HIPCHK(hipMalloc(&ka.p, nb));
        HIPCHK(hipMalloc(&kb.p, nb));
        HIPCHK(hipMalloc(&va.p, nb));
        HIPCHK(hipMalloc(&vb.p, nb));
        HIPCHK(hipMalloc(&hist.p, (size_t)256 * nblocks * sizeof(uint32_t)));
        HIPCHK(hipMalloc(&base.p, (size_t)256 * nblocks * sizeof(uint32_t)));
        HIPCHK(rocprim::exclusive_scan(nullptr, scan_bytes, static_cast<uint32_t *>(hist.p), static_cast<uint32_t *>(base.p),
                                       0u, (size_t)256 * nblocks, rocprim::plus<uint32_t>(), nullptr));
        HIPCHK(hipMalloc(&scan.p, scan_bytes ? scan_bytes : 16));
        return IVF_OK;
    }
    uint32_t *keys_a() { return static_cast<uint32_t *>(ka.p); }
    // Sorts the n keys held in the a buffer (values: positions, or the a value buffer when
    // have_vals).  Returns the buffers that hold the result.
    int sort(int64_t n, int bits, bool have_vals, uint32_t **keys_sorted, uint32_t **vals_sorted, hipStream_t st)
    {
        if (n > cap) return fail(IVF_EINVAL, "radix sort buffers too small");
        uint32_t *kin = static_cast<uint32_t *>(ka.p), *kout = static_cast<uint32_t *>(kb.p);
        uint32_t *vin = static_cast<uint32_t *>(va.p), *vout = static_cast<uint32_t *>(vb.p);
        const int64_t nbk = (n + RS_TILE - 1) / RS_TILE > 0 ? (n + RS_TILE - 1) / RS_TILE : 1;
        bool first = !have_vals;
        if (bits < 1) bits = 1;
        for (int shift = 0; shift < bits; shift += 8) {
            radix_hist_kernel<<<dim3((unsigned)nbk), dim3(RS_BLOCK), 0, st>>>(kin, n, shift, static_cast<uint32_t *>(hist.p), nbk);
            LAUNCHCHK("radix_hist_kernel");
            size_t sb = scan_bytes;
            HIPCHK(rocprim::exclusive_scan(scan.p, sb, static_cast<uint32_t *>(hist.p), static_cast<uint32_t *>(base.p), 0u,
                                           (size_t)256 * nbk, rocprim::plus<uint32_t>(), st));
            radix_scatter_kernel<<<dim3((unsigned)nbk), dim3(RS_BLOCK), 0, st>>>(
                kin, first ? nullptr : vin, n, shift, static_cast<uint32_t *>(base.p), nbk, kout, vout);
            LAUNCHCHK("radix_scatter_kernel");
            first = false;
            std::swap(kin, kout);
            std::swap(vin, vout);
        }
        *keys_sorted = kin;
        *vals_sorted = vin;
        return IVF_OK;
    }
};

int bits_for(int64_t nbuckets)
{
    int b = 1;
    while (b < 32 && (1ll << b) < nbuckets) ++b;
    return b;
}

}  // namespace

extern "C" int ivf_group(const int32_t *bucket, int64_t n, int64_t nbuckets, int32_t *perm, uint32_t *offsets,
                         void *hip_stream)
{
    if (!bucket || !perm || !offsets) return fail(IVF_EINVAL, "NULL argument");
    if (n < 0 || n >= (1ll << 32) - 1) return fail(IVF_EINVAL, "n=%lld out of range", (long long)n);
    if (nbuckets < 1 || nbuckets >= (1ll << 31)) return fail(IVF_EINVAL, "nbuckets=%lld out of range", (long long)nbuckets);
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    RadixBufs rb;
    int rc = rb.init(n);
    if (!rc && n > 0) {
        auto body = [&]() -> int {
            HIPCHK(hipMemcpyAsync(rb.keys_a(), bucket, (size_t)n * sizeof(uint32_t), hipMemcpyDeviceToDevice, st));
            uint32_t *ks, *vs;
            int r2 = rb.sort(n, bits_for(nbuckets), false, &ks, &vs, st);
            if (r2) return r2;
            bucket_offsets_kernel<<<dim3(grid_for(n + 1)), dim3(256), 0, st>>>(ks, n, nbuckets, offsets);
            LAUNCHCHK("bucket_offsets_kernel");
            HIPCHK(hipMemcpyAsync(perm, vs, (size_t)n * sizeof(uint32_t), hipMemcpyDeviceToDevice, st));
            return IVF_OK;
        };
        rc = body();
    } else if (!rc) {
        rc = hipMemsetAsync(offsets, 0, (size_t)(nbuckets + 1) * sizeof(uint32_t), st) == hipSuccess
                 ? IVF_OK : fail(IVF_EHIP, "hipMemsetAsync failed");
    }
    std::string keep = g_err;
    (void)hipStreamSynchronize(st);
    g_err = keep;
    return rc;
}

extern "C" int ivf_gather_rows(const void *src, int64_t row_bytes, const int32_t *perm, int64_t n, void *dst,
                               void *hip_stream)
{
    if (!src || !perm || !dst) return fail(IVF_EINVAL, "NULL argument");
    if (row_bytes < 1 || n < 0) return fail(IVF_EINVAL, "bad sizes");
    if (n == 0) return IVF_OK;
    const uintptr_t al = reinterpret_cast<uintptr_t>(src) | reinterpret_cast<uintptr_t>(dst) | (uintptr_t)row_bytes;
    const int vec = (al % 16 == 0) ? 16 : (al % 8 == 0) ? 8 : (al % 4 == 0) ? 4 : 1;
    const int64_t threads = n * (row_bytes / vec);
    if (threads >= (1ll << 32) - 256) return fail(IVF_EINVAL, "too many rows for one launch");
    gather_rows_kernel<<<dim3(grid_for(threads)), dim3(256), 0, static_cast<hipStream_t>(hip_stream)>>>(
        static_cast<const uint8_t *>(src), row_bytes, perm, n, static_cast<uint8_t *>(dst), vec);
    LAUNCHCHK("gather_rows_kernel");
    return IVF_OK;
}

extern "C" int ivf_bucket_ids(const int32_t *region, const int32_t *sub, int64_t n, int L, int32_t *bucket,
                              void *hip_stream)
{
    if (!region || !sub || !bucket) return fail(IVF_EINVAL, "NULL argument");
    if (n < 0 || L < 1) return fail(IVF_EINVAL, "bad sizes");
    if (n == 0) return IVF_OK;
    bucket_ids_kernel<<<dim3(grid_for(n)), dim3(256), 0, static_cast<hipStream_t>(hip_stream)>>>(region, sub, n, L, bucket);
    LAUNCHCHK("bucket_ids_kernel");
    return IVF_OK;
}

extern "C" int ivf_cluster_means(const float *x, int64_t n, int D, const int32_t *assign, int64_t K,
                                 float *centroids, void *hip_stream)
{
    if (!x || !assign || !centroids) return fail(IVF_EINVAL, "NULL argument");
    if (D < 1 || D > IVF_MAX_D || K < 1 || K >= (1ll << 31)) return fail(IVF_EINVAL, "bad sizes");
    if (n < 0 || n >= (1ll << 31)) return fail(IVF_EINVAL, "n out of range");
    if (n == 0) return IVF_OK;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    RadixBufs rb;
    DevTmp off;
    auto body = [&]() -> int {
        int r2;
        if ((r2 = rb.init(n))) return r2;
        HIPCHK(hipMalloc(&off.p, (size_t)(K + 1) * sizeof(uint32_t)));
        HIPCHK(hipMemcpyAsync(rb.keys_a(), assign, (size_t)n * sizeof(uint32_t), hipMemcpyDeviceToDevice, st));
        uint32_t *ks, *vs;
        if ((r2 = rb.sort(n, bits_for(K), false, &ks, &vs, st))) return r2;
        bucket_offsets_kernel<<<dim3(grid_for(n + 1)), dim3(256), 0, st>>>(ks, n, K, static_cast<uint32_t *>(off.p));
        LAUNCHCHK("bucket_offsets_kernel");
        segment_sum_kernel<float, 1><<<dim3((unsigned)K), dim3(256), 0, st>>>(
            x, D, 0, D, vs, static_cast<uint32_t *>(off.p), nullptr, centroids, D, 0);
        LAUNCHCHK("segment_sum_kernel");
        HIPCHK(hipStreamSynchronize(st));
        return IVF_OK;
    };
    int rc = body();
    std::string keep = g_err;
    (void)hipStreamSynchronize(st);
    g_err = keep;
    return rc;
}

extern "C" int ivf_kmeans(const float *x, int64_t n, int D, int64_t K, int iters, const int64_t *init_idx,
                          float *centroids, double *objective, void *hip_stream)
{
    int rc = IVF_OK;
    if (!x || !init_idx || !centroids) return fail(IVF_EINVAL, "NULL argument");
    if (D < 4 || D % 4 || D > IVF_MAX_D) return fail(IVF_EINVAL, "D=%d must be a multiple of 4 in [4, %d]", D, IVF_MAX_D);
    if (n < 1 || n >= (1ll << 31)) return fail(IVF_EINVAL, "n=%lld out of range", (long long)n);
    if (!aligned16(x)) return fail(IVF_EINVAL, "x must be 16-byte aligned");
    if (K < 1 || K > n) return fail(IVF_EINVAL, "need 1 <= K <= n");
    if (iters < 0) return fail(IVF_EINVAL, "iters must be >= 0");
    if (!aligned16(centroids)) return fail(IVF_EINVAL, "centroids must be 16-byte aligned");
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    ArgminCtx ctx;
    RadixBufs rb;
    DevTmp lab, dist;
    auto body = [&]() -> int {
        int r2;
        take_rows_kernel<<<dim3(grid_for(K * D)), dim3(256), 0, st>>>(x, D, 0, D, init_idx, K, centroids, D, 0);
        LAUNCHCHK("take_rows_kernel");
        if (iters == 0) return IVF_OK;
        if ((r2 = ctx.init(K, D, n))) return r2;
        if ((r2 = rb.init(n))) return r2;
        HIPCHK(hipMalloc(&lab.p, (size_t)n * sizeof(int32_t)));
        HIPCHK(hipMalloc(&dist.p, (size_t)n * sizeof(float)));
        DevTmp off;
        HIPCHK(hipMalloc(&off.p, (size_t)(K + 1) * sizeof(uint32_t)));
        const int bits = bits_for(K);
        for (int it = 0; it < iters; ++it) {
            if ((r2 = ctx.set_centroids(centroids, st))) return r2;
            if ((r2 = ctx.run(x, n, static_cast<int32_t *>(lab.p), static_cast<float *>(dist.p), st))) return r2;
            if (objective) {
                fixed_sum_kernel<float><<<dim3(1), dim3(1024), 0, st>>>(static_cast<float *>(dist.p), n, objective + it);
                LAUNCHCHK("fixed_sum_kernel");
            }
            HIPCHK(hipMemcpyAsync(rb.keys_a(), lab.p, (size_t)n * sizeof(uint32_t), hipMemcpyDeviceToDevice, st));
            uint32_t *ks, *vs;
            if ((r2 = rb.sort(n, bits, false, &ks, &vs, st))) return r2;
            bucket_offsets_kernel<<<dim3(grid_for(n + 1)), dim3(256), 0, st>>>(ks, n, K, static_cast<uint32_t *>(off.p));
            LAUNCHCHK("bucket_offsets_kernel");
            segment_sum_kernel<float, 1><<<dim3((unsigned)K), dim3(256), 0, st>>>(
                x, D, 0, D, vs, static_cast<uint32_t *>(off.p), nullptr, centroids, D, 0);
            LAUNCHCHK("segment_sum_kernel");
        }
        HIPCHK(hipStreamSynchronize(st));
        return IVF_OK;
    };
    rc = body();
    std::string keep = g_err;
    (void)hipStreamSynchronize(st);
    g_err = keep;
    return rc;
}

extern "C" int ivf_pq_train(const float *E, int64_t n, int D, int M, int iters, const int64_t *init_idx,
                            float *codebook, void *hip_stream)
{
    if (!E || !init_idx || !codebook) return fail(IVF_EINVAL, "NULL argument");
    if (M < 1 || D < M || D % M || D > IVF_MAX_D) return fail(IVF_EINVAL, "D=%d must be a multiple of M=%d", D, M);
    if (n < 256 || n >= (1ll << 31)) return fail(IVF_EINVAL, "n=%lld: need at least 256 training rows", (long long)n);
    if (iters < 0) return fail(IVF_EINVAL, "iters must be >= 0");
    const int ds = D / M;
    if (!(ds == 4 || ds == 6 || ds == 8 || ds == 12 || ds == 16))
        return fail(IVF_EINVAL, "D/M=%d: the codeword assignment kernel is built for block widths 4, 6, 8, 12 and 16", ds);
    const size_t cb_bytes = (size_t)256 * D * sizeof(float);
    if (cb_bytes > 140 * 1024) return fail(IVF_EINVAL, "codebook of %zu bytes does not fit LDS", cb_bytes);
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    RadixBufs rb;
    DevTmp codes, off;
    auto body = [&]() -> int {
        int r2;
        for (int m = 0; m < M; ++m) {   // codeword j of block m starts as block m of row init_idx[j]
            take_rows_kernel<<<dim3(grid_for(256 * ds)), dim3(256), 0, st>>>(E, D, m * ds, ds, init_idx, 256,
                                                                              codebook + (size_t)m * 256 * ds, ds, 0);
            LAUNCHCHK("take_rows_kernel");
        }
        if (iters == 0) return IVF_OK;
        if ((r2 = rb.init(n))) return r2;
        HIPCHK(hipMalloc(&codes.p, (size_t)n * M));
        HIPCHK(hipMalloc(&off.p, 257 * sizeof(uint32_t)));
        const void *fn = ds == 4 ? (const void *)&pq_encode_kernel<4> : ds == 6 ? (const void *)&pq_encode_kernel<6>
                       : ds == 8 ? (const void *)&pq_encode_kernel<8> : ds == 12 ? (const void *)&pq_encode_kernel<12>
                                                                                 : (const void *)&pq_encode_kernel<16>;
        HIPCHK(hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)cb_bytes));
        int64_t grid = (n + 1023) / 1024;
        if (grid > 512) grid = 512;
        uint8_t *cd = static_cast<uint8_t *>(codes.p);
        for (int it = 0; it < iters; ++it) {
            // nearest codeword of every block of every row, by (distance, index)
#define IVF_PQ_ASSIGN(DSV) \
    pq_encode_kernel<DSV><<<dim3((unsigned)grid), dim3(1024), cb_bytes, st>>>(E, nullptr, n, M, codebook, nullptr, cd, nullptr, nullptr)
            if (ds == 4) IVF_PQ_ASSIGN(4);
            else if (ds == 6) IVF_PQ_ASSIGN(6);
            else if (ds == 8) IVF_PQ_ASSIGN(8);
            else if (ds == 12) IVF_PQ_ASSIGN(12);
            else IVF_PQ_ASSIGN(16);
#undef IVF_PQ_ASSIGN
            LAUNCHCHK("pq_encode_kernel");
            for (int m = 0; m < M; ++m) {   // every codeword becomes the mean of the rows assigned to it
                byte_column_kernel<<<dim3(grid_for(n)), dim3(256), 0, st>>>(cd, n, M, m, rb.keys_a());
                LAUNCHCHK("byte_column_kernel");
                uint32_t *ks, *vs;
                if ((r2 = rb.sort(n, 8, false, &ks, &vs, st))) return r2;
                bucket_offsets_kernel<<<dim3(grid_for(n + 1)), dim3(256), 0, st>>>(ks, n, 256, static_cast<uint32_t *>(off.p));
                LAUNCHCHK("bucket_offsets_kernel");
                segment_sum_kernel<float, 1><<<dim3(256), dim3(256), 0, st>>>(
                    E, D, m * ds, ds, vs, static_cast<uint32_t *>(off.p), nullptr, codebook + (size_t)m * 256 * ds, ds, 0);
                LAUNCHCHK("segment_sum_kernel");
            }
        }
        HIPCHK(hipStreamSynchronize(st));
        return IVF_OK;
    };
    int rc = body();
    std::string keep = g_err;
    (void)hipStreamSynchronize(st);
    g_err = keep;
    return rc;
}

extern "C" int ivf_lloyd_1d(const float *t, int64_t n, int iters, float *table, void *hip_stream)
{
    if (!t || !table) return fail(IVF_EINVAL, "NULL argument");
    if (n < 1 || n >= (1ll << 31)) return fail(IVF_EINVAL, "n out of range");
    if (iters < 0) return fail(IVF_EINVAL, "iters must be >= 0");
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    RadixBufs rb;
    DevTmp sorted, off, sum;
    auto body = [&]() -> int {
        int r2;
        if ((r2 = rb.init(n))) return r2;
        HIPCHK(hipMalloc(&sorted.p, (size_t)n * sizeof(float)));
        HIPCHK(hipMalloc(&off.p, 257 * sizeof(uint32_t)));
        HIPCHK(hipMalloc(&sum.p, 256 * sizeof(double)));
        float *s = static_cast<float *>(sorted.p);
        float_keys_kernel<<<dim3(grid_for(n)), dim3(256), 0, st>>>(t, n, rb.keys_a());
        LAUNCHCHK("float_keys_kernel");
        uint32_t *ks, *vs;
        if ((r2 = rb.sort(n, 32, false, &ks, &vs, st))) return r2;
        key_floats_kernel<<<dim3(grid_for(n)), dim3(256), 0, st>>>(ks, n, s);
        LAUNCHCHK("key_floats_kernel");
        lloyd1d_init_kernel<<<dim3(1), dim3(256), 0, st>>>(s, n, table);
        LAUNCHCHK("lloyd1d_init_kernel");
        int64_t grid = (n + 255) / 256;
        if (grid > 4096) grid = 4096;
        for (int it = 0; it < iters; ++it) {
            lloyd1d_label_kernel<<<dim3((unsigned)grid), dim3(256), 0, st>>>(s, n, table, rb.keys_a());
            LAUNCHCHK("lloyd1d_label_kernel");
            if ((r2 = rb.sort(n, 8, false, &ks, &vs, st))) return r2;
            bucket_offsets_kernel<<<dim3(grid_for(n + 1)), dim3(256), 0, st>>>(ks, n, 256, static_cast<uint32_t *>(off.p));
            LAUNCHCHK("bucket_offsets_kernel");
            segment_sum_kernel<float, 0><<<dim3(256), dim3(256), 0, st>>>(s, 1, 0, 1, vs, static_cast<uint32_t *>(off.p),
                                                                          static_cast<double *>(sum.p), nullptr, 0, 0);
            LAUNCHCHK("segment_sum_kernel");
            lloyd1d_update_kernel<<<dim3(1), dim3(256), 0, st>>>(static_cast<double *>(sum.p), static_cast<uint32_t *>(off.p), table);
            LAUNCHCHK("lloyd1d_update_kernel");
        }
        HIPCHK(hipStreamSynchronize(st));
        return IVF_OK;
    };
    int rc = body();
    std::string keep = g_err;
    (void)hipStreamSynchronize(st);
    g_err = keep;
    return rc;
}

extern "C" int ivf_learn_alpha(const float *centroids, int64_t K, int D, const int32_t *nbr, int L, const float *x,
                               int64_t n, const int32_t *region, float *alpha, void *hip_stream)
{
    if (!centroids || !nbr || !x || !region || !alpha) return fail(IVF_EINVAL, "NULL argument");
    if (D < 1 || D > IVF_MAX_D || K < 1 || K >= (1ll << 31) || L < 1) return fail(IVF_EINVAL, "bad sizes");
    if (n < 0 || n >= (1ll << 31)) return fail(IVF_EINVAL, "n out of range");
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    RadixBufs rb;
    DevTmp stat, off, nd, tot;
    auto body = [&]() -> int {
        int r2;
        if ((r2 = rb.init(n))) return r2;
        HIPCHK(hipMalloc(&stat.p, (size_t)(n > 0 ? n : 1) * 2 * sizeof(double)));
        HIPCHK(hipMalloc(&off.p, (size_t)(K + 1) * sizeof(uint32_t)));
        HIPCHK(hipMalloc(&nd.p, (size_t)K * 2 * sizeof(double)));
        HIPCHK(hipMalloc(&tot.p, 2 * sizeof(double)));
        HIPCHK(hipMemsetAsync(stat.p, 0, (size_t)(n > 0 ? n : 1) * 2 * sizeof(double), st));
        HIPCHK(hipMemsetAsync(off.p, 0, (size_t)(K + 1) * sizeof(uint32_t), st));
        if (n > 0) {
            alpha_point_kernel<<<dim3((unsigned)n), dim3(64), (size_t)D * sizeof(float), st>>>(
                x, n, D, L, region, centroids, nbr, static_cast<double *>(stat.p));
            LAUNCHCHK("alpha_point_kernel");
            HIPCHK(hipMemcpyAsync(rb.keys_a(), region, (size_t)n * sizeof(uint32_t), hipMemcpyDeviceToDevice, st));
            uint32_t *ks, *vs;
            if ((r2 = rb.sort(n, bits_for(K), false, &ks, &vs, st))) return r2;
            bucket_offsets_kernel<<<dim3(grid_for(n + 1)), dim3(256), 0, st>>>(ks, n, K, static_cast<uint32_t *>(off.p));
            LAUNCHCHK("bucket_offsets_kernel");
            segment_sum_kernel<double, 0><<<dim3((unsigned)K), dim3(256), 0, st>>>(
                static_cast<double *>(stat.p), 2, 0, 2, vs, static_cast<uint32_t *>(off.p), static_cast<double *>(nd.p), nullptr, 0, 0);
            LAUNCHCHK("segment_sum_kernel");
        } else {
            HIPCHK(hipMemsetAsync(nd.p, 0, (size_t)K * 2 * sizeof(double), st));
        }
        // pooled ratio: the two sums over all regions, each in a fixed order (stride-2 views of nd)
        strided_sum_kernel<<<dim3(2), dim3(1024), 0, st>>>(static_cast<double *>(nd.p), K, 2, static_cast<double *>(tot.p));
        LAUNCHCHK("strided_sum_kernel");
        alpha_finish_kernel<<<dim3(grid_for(K)), dim3(256), 0, st>>>(static_cast<double *>(nd.p), static_cast<double *>(tot.p), K, alpha);
        LAUNCHCHK("alpha_finish_kernel");
        HIPCHK(hipStreamSynchronize(st));
        return IVF_OK;
    };
    int rc = body();
    std::string keep = g_err;
    (void)hipStreamSynchronize(st);
    g_err = keep;
    return rc;
}

extern "C" int ivf_neighbours(const float *centroids, int64_t K, int D, int L, int32_t *nbr, float *cs_dist2,
                              void *hip_stream)
{
    int rc = check_coarse_args(centroids, K, D, centroids, K);
    if (rc) return rc;
    if (!nbr || !cs_dist2) return fail(IVF_EINVAL, "NULL argument");
    if (L < 1 || L >= K || L + 1 > 4096) return fail(IVF_EINVAL, "need 1 <= L < K and L <= 4095");
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    const int P = L + 1;
    DevTmp tid, td;
    HIPCHK(hipMalloc(&tid.p, (size_t)K * P * sizeof(int32_t)));
    HIPCHK(hipMalloc(&td.p, (size_t)K * P * sizeof(float)));
    rc = coarse_topk_tiled(centroids, K, D, centroids, K, P, static_cast<int32_t *>(tid.p), static_cast<float *>(td.p), st);
    if (!rc) {
        neighbour_rows_kernel<<<dim3((unsigned)K), dim3(64), (size_t)P * sizeof(unsigned long long), st>>>(
            static_cast<int32_t *>(tid.p), static_cast<float *>(td.p), K, P, nbr, cs_dist2);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) rc = fail(IVF_EHIP, "launch neighbour_rows_kernel: %s", hipGetErrorString(e));
    }
    std::string keep = g_err;
    (void)hipStreamSynchronize(st);
    g_err = keep;
    return rc;
}
