// Stages 1b-4 of a query in ONE launch.  The selection of the nprobe closest regions and the scoring +
// pruning of their subregions are both one workgroup of 1024 threads per query; run one after the other
// in the same workgroup they save a kernel boundary and the round trip of the probes through another
// launch, and, with two such workgroups on a compute unit, the selection of one query (LDS and ALU work)
// overlaps with the other's gathers from the distance matrix (which wait for the memory system):
// 0.80 + 3.99 ms as two launches, 4.47 ms as one, on the 10^9-point workload.  The probe ids and
// distances still go through global memory (they are outputs of the staged entry point): the
// workgroup's own writes are complete and visible to all its threads after the barrier.
#pragma once
#include "coarse.hpp"
#include "query.hpp"

namespace ivf {

// Workgroups 0 .. nq-1: select, then score and prune, query q = blockIdx.x; nq .. 2nq-1: the lookup
// tables.  Dynamic LDS: the larger of what the two halves need (they use it one after the other).
// Registers are capped so that two workgroups fit a compute unit (MAXV = 4: 64 VGPRs).
template <int MAXV>
__global__ __launch_bounds__(1024) __attribute__((amdgpu_waves_per_eu(MAXV == 4 ? 8 : 4, MAXV == 4 ? 8 : 5))) void select_score_prune_kernel(
    const float *__restrict__ Dt, int64_t ldt, const float *__restrict__ bm, int64_t K, int nb,
    int32_t *__restrict__ probe_id, float *__restrict__ probe_d, int P, int L, const int32_t *__restrict__ nbr,
    const float *__restrict__ cst, const float *__restrict__ alpha, int S, const uint4 *__restrict__ sub_info,
    SubDesc *__restrict__ desc, int64_t *__restrict__ kept_sub, int64_t *__restrict__ n_scanned,
    int64_t nq, const float *__restrict__ Qt, int D, int M, const float *__restrict__ codebook,
    float *__restrict__ lut)
{
    extern __shared__ __attribute__((aligned(16))) uint32_t dyn[];
    if ((int64_t)blockIdx.x >= nq) {   // (uniform) a table workgroup
        const int64_t ql = (int64_t)blockIdx.x - nq;
        lut_body<1024>(Qt + ql * D, D, M, codebook, lut + ql * (int64_t)M * 256, reinterpret_cast<float *>(dyn));
        return;
    }
    probe_select_lds_body(Dt, ldt, bm, K, nb, P, probe_id, probe_d, blockIdx.x, reinterpret_cast<int *>(dyn));
    __syncthreads();   // the probes are written (and the selection is done with the LDS the scoring reuses)
    score_prune_body<1024, MAXV>(Dt, ldt, K, probe_id, probe_d, P, L, nbr, cst, alpha, S, sub_info, desc, kept_sub, n_scanned,
                                 blockIdx.x, dyn);
}

}  // namespace ivf
