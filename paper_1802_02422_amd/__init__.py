"""MI355X-native batched query path of the inverted index with grouping and pruning.

The work is done by hand-written gfx950 HIP kernels behind the C ABI declared in
``include/ivf_gp.h``; this package is the thin ctypes binding over it (argument
marshalling only).  There is no CPU fallback: without the built library every call
raises.
"""
from .binding import (  # noqa: F401
    IvfError,
    IndexDesc,
    library_path,
    load_library,
    ivf_load_index,
    ivf_free_index,
    ivf_set_scratch_limit,
    ivf_search,
    ivf_search_stages,
    ivf_search_noalloc,
    ivf_search_budget,
    ivf_num_kept,
    ivf_coarse_topk,
    ivf_assign_stats,
    ivf_encode,
    ivf_rotate,
    ivf_kmeans,
    ivf_cluster_means,
    ivf_bucket_ids,
    ivf_neighbours,
    ivf_learn_alpha,
    ivf_pq_train,
    ivf_lloyd_1d,
    ivf_group,
    ivf_gather_rows,
    ivf_last_error,
    ivf_profile_enable,
    ivf_copy_bytes,
    ivf_profile_read,
    STAGE_NAMES,
)
