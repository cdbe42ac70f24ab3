// Grouping of a batch by expert: sequences are sorted by (expert id, sequence
// index) and cut into row tiles that never span two sequences, so every tile
// has exactly one adapter (Section 1: one expert per query; Section 4.1: id -1
// = no adapter, base model only).  For small batches the tokens themselves are
// also grouped by expert, so that the decode kernels read each distinct
// adapter once.  Everything happens on the device in one workgroup: the host
// never looks at the ids.  Offsets that do not tile [0, T) in order make the
// whole batch base-only (and raise the sticky fault): every output row is still
// written.
#include "kernels.h"
#include "plan_body.h"

namespace moin {

template <int PLAN_THREADS>
__global__ __launch_bounds__(PLAN_THREADS) void plan_kernel(PlanView pv, const int *seq_offsets,
                                                            const int *expert_ids, const int *rank_of_expert,
                                                            int *err_word)
{
    plan_body<PLAN_THREADS>(pv, seq_offsets, expert_ids, rank_of_expert, err_word);
}

hipError_t launch_plan(const PlanView &pv, const int *seq_offsets, const int *expert_ids,
                       const int *rank_of_expert, int *err_word, hipStream_t stream)
{
    if (pv.S <= 2 * PLAN_THREADS_SMALL)
        hipLaunchKernelGGL(plan_kernel<PLAN_THREADS_SMALL>, dim3(1), dim3(PLAN_THREADS_SMALL), 0, stream, pv,
                           seq_offsets, expert_ids, rank_of_expert, err_word);
    else
        hipLaunchKernelGGL(plan_kernel<PLAN_THREADS_MAX>, dim3(1), dim3(PLAN_THREADS_MAX), 0, stream, pv,
                           seq_offsets, expert_ids, rank_of_expert, err_word);
    return hipGetLastError();
}

}  // namespace moin
