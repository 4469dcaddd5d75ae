// Alg. 1 taken literally for M <= 16: pull toward a supplied consensus variable, push along the
// pulled gap away from the workers' average or from the consensus variable.
#include "dppf_internal.h"

namespace dppf_detail {
namespace {

template <int REF>
int reduce(dppf_plan* p, const void** xp, const void** xcp, float pull, GridShape* shape, hipStream_t s) {
  float* const* x = (float* const*)(xp);
  const float* const* xc = (const float* const*)(xcp);
  const float keep = static_cast<float>(1.0 - static_cast<double>(pull));
  DPPF_SWITCH_M(p->M, {
    constexpr int kU = unroll_seq(kM);
    auto kern = k_seq1<kM, kU, REF>;
    int grid = 0, gfull = 0;
    const int rc = grid_for(p, p->sweep, kern, 1, 1, kBlocksPerCUReadOnly, 0, &gfull, &grid);
    if (rc) return rc;
    const Walk walk = plan_walk(p, p->sweep, gfull, 1, 1, dppf_walk::kEvenSplit, 0.0);
    if (!rows_fit(p, grid, walk)) return DPPF_ELIMIT;
    shape->grid = grid;
    shape->walk = walk;
    hipLaunchKernelGGL(kern, dim3(grid), dim3(kBlock), 0, s, p->sweep.dev, walk, p->T, x, xc, pull, keep,
                       p->partials, p->partials_rows);
  })
  HIP_TRY(hipGetLastError());
  return DPPF_OK;
}

template <int REF>
int update(dppf_plan* p, const void** xp, const void** xcp, float pull, float push, int nparts, float* r_post_out,
           hipStream_t s) {
  float* const* x = (float* const*)(xp);
  const float* const* xc = (const float* const*)(xcp);
  const float keep = static_cast<float>(1.0 - static_cast<double>(pull));
  DPPF_SWITCH_M(p->M, {
    constexpr int kU = unroll_seq(kM);
    auto kern = k_seq2<kM, kU, REF>;
    int grid = 0, gfull = 0;
    const int rc = grid_for(p, p->sweep, kern, 1, 1, kBlocksPerCUReadWrite, 0, &gfull, &grid);
    if (rc) return rc;
    const Walk walk = plan_walk(p, p->sweep, gfull, 1, 1, dppf_walk::kOnDemand, 8.0 * kM + 4.0);
    hipLaunchKernelGGL(kern, dim3(grid), dim3(kBlock), 0, s, p->sweep.dev, walk, p->T, x, xc, pull, keep, push,
                       p->partials, nparts, p->partials_rows, r_post_out);
  })
  HIP_TRY(hipGetLastError());
  return DPPF_OK;
}

}  // namespace

int launch_seq_reduce(dppf_plan* p, const void** xp, const void** xcp, bool from_consensus, float pull,
                      GridShape* shape, hipStream_t s) {
  return from_consensus ? reduce<1>(p, xp, xcp, pull, shape, s) : reduce<0>(p, xp, xcp, pull, shape, s);
}

int launch_seq_update(dppf_plan* p, const void** xp, const void** xcp, bool from_consensus, float pull, float push,
                      int nparts, float* r_post_out, hipStream_t s) {
  return from_consensus ? update<1>(p, xp, xcp, pull, push, nparts, r_post_out, s)
                        : update<0>(p, xp, xcp, pull, push, nparts, r_post_out, s);
}

}  // namespace dppf_detail
