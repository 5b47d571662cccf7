/* Compiled as C99 against include/ivf_gp.h and linked with the built library: every call below
 * goes through the real prototypes, so a signature that drifts between header and library fails to
 * compile or link.  It exercises only what needs no GPU: the host-only entry point and the
 * argument checks, which must return IVF_EINVAL (and set a message) before any device work. */
#include <stdio.h>
#include <string.h>
#include "ivf_gp.h"

#define EXPECT(cond)                                                     \
    do {                                                                 \
        if (!(cond)) { printf("FAILED line %d: %s\n", __LINE__, #cond); return 1; } \
    } while (0)

int main(void)
{
    ivf_index *ix = NULL;
    ivf_index_desc d;
    float buf[4] = {0};
    int32_t ib[4] = {0};
    uint8_t ub[4] = {0};
    int64_t lb[4] = {0};
    uint32_t u32[4] = {0};
    double db[4] = {0};
    memset(&d, 0, sizeof d);

    EXPECT(ivf_num_kept(256, 64, 0.2f) == 3277);
    EXPECT(ivf_num_kept(16, 8, 0.5f) == 64);
    EXPECT(ivf_num_kept(3, 5, 1e-9f) == 1);
    EXPECT(ivf_num_kept(3, 5, 1.0f) == 15);

    EXPECT(ivf_load_index(NULL, NULL, &ix) == IVF_EINVAL);
    EXPECT(strlen(ivf_last_error()) > 0);
    d.D = 6; d.M = 8; d.L = 1; d.K = 4; d.N = 0;                 /* D not a multiple of 4 */
    EXPECT(ivf_load_index(&d, NULL, &ix) == IVF_EINVAL && ix == NULL);
    d.D = 96; d.M = 7;                                           /* unsupported code length */
    EXPECT(ivf_load_index(&d, NULL, &ix) == IVF_EINVAL);
    d.M = 8;                                                     /* arrays missing */
    EXPECT(ivf_load_index(&d, NULL, &ix) == IVF_EINVAL);
    EXPECT(ivf_set_scratch_limit(NULL, 1 << 20) == IVF_EINVAL);
    EXPECT(ivf_search(NULL, buf, 1, 1, 0.5f, 1, ib, buf, NULL) == IVF_EINVAL);
    EXPECT(ivf_search_noalloc(NULL, buf, 1, 1, 0.5f, 1, ib, buf, NULL) == IVF_EINVAL);
    EXPECT(ivf_search_stages(NULL, buf, 1, 1, 0.5f, 1, ib, buf, ib, buf, lb, lb, NULL) == IVF_EINVAL);
    EXPECT(ivf_search_budget(NULL, buf, 1, 1, 0.5f, 100, 1, ib, buf, lb, ub, lb, NULL) == IVF_EINVAL);
    EXPECT(ivf_search_budget(NULL, buf, 1, 1, 0.5f, 0, 1, ib, buf, lb, ub, lb, NULL) == IVF_EINVAL);
    EXPECT(ivf_coarse_topk(NULL, 4, 96, buf, 1, 1, ib, buf, NULL) == IVF_EINVAL);
    EXPECT(ivf_coarse_topk(buf, 4, 6, buf, 1, 1, ib, buf, NULL) == IVF_EINVAL);
    EXPECT(ivf_encode(NULL, buf, 1, NULL, ib, ib, ub, ub, buf, buf, NULL) == IVF_EINVAL);
    EXPECT(ivf_rotate(NULL, 1, 4, buf, buf, NULL) == IVF_EINVAL);
    EXPECT(ivf_kmeans(NULL, 10, 4, 2, 1, lb, buf, db, NULL) == IVF_EINVAL);
    EXPECT(ivf_cluster_means(NULL, 1, 4, ib, 1, buf, NULL) == IVF_EINVAL);
    EXPECT(ivf_neighbours(NULL, 4, 4, 1, ib, buf, NULL) == IVF_EINVAL);
    EXPECT(ivf_learn_alpha(NULL, 4, 4, ib, 1, buf, 1, ib, buf, NULL) == IVF_EINVAL);
    EXPECT(ivf_pq_train(NULL, 1000, 96, 8, 1, lb, buf, NULL) == IVF_EINVAL);
    EXPECT(ivf_lloyd_1d(NULL, 10, 1, buf, NULL) == IVF_EINVAL);
    EXPECT(ivf_group(NULL, 1, 1, ib, u32, NULL) == IVF_EINVAL);
    EXPECT(ivf_bucket_ids(NULL, ib, 1, 1, ib, NULL) == IVF_EINVAL);
    EXPECT(ivf_gather_rows(NULL, 4, ib, 1, buf, NULL) == IVF_EINVAL);
    EXPECT(ivf_copy_bytes(NULL, buf, 16, NULL) == IVF_EINVAL);
    EXPECT(ivf_profile_enable(NULL, 1) == IVF_EINVAL);
    EXPECT(ivf_profile_read(NULL, db, lb) == IVF_EINVAL);
    ivf_free_index(NULL);                                        /* a no-op */
    EXPECT(IVF_N_STAGES == 6 && IVF_MAX_SCORES == 32768 && IVF_NOALLOC_SCRATCH_BYTES == (64 << 20));
    printf("abi ok\n");
    return 0;
}
