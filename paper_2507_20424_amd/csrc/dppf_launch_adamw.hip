// AdamW local step (one worker at a time) and sweep 1 of the round with the AdamW step folded in
// (M <= 16).
#include "dppf_internal.h"

namespace dppf_detail {

int launch_adamw_step(dppf_plan* p, const void** xd, const void** ad, const void** sd, const void** gd,
                      const AdamHyper hp, hipStream_t s) {
  auto kern = k_adamw_step<2>;
  int grid = 0, gfull = 0, rc;
  if ((rc = grid_for(p, p->step, kern, p->M, kTilesPerWorkerItem, kBlocksPerCUReadWrite, 0, &gfull, &grid))) return rc;
  if ((rc = timing_begin(p, DPPF_K_ADAMW_STEP, s))) return rc;
  const Walk walk = plan_walk(p, p->step, gfull, p->M, kTilesPerWorkerItem, dppf_walk::kOnDemand, 28.0);
  hipLaunchKernelGGL(kern, dim3(grid), dim3(kBlock), 0, s, p->step.dev, walk, p->M, p->T, (float* const*)(xd),
                     (float* const*)(ad), (float* const*)(sd), (const float* const*)(gd), hp);
  HIP_TRY(hipGetLastError());
  return timing_end(p, s);
}

int launch_adamw_reduce(dppf_plan* p, const void** xd, const void** ad, const void** sd, const void** gd,
                        const AdamHyper hp, GridShape* shape, hipStream_t s) {
  DPPF_SWITCH_M(p->M, {
    constexpr int kU = unroll_fused(kM);
    auto kern = k_adamw_reduce<kM, kU>;
    int gfull = 0, grid = 0;
    const int rc = grid_for(p, p->sweep, kern, 1, 1, kBlocksPerCUReadWrite, 0, &gfull, &grid);
    if (rc) return rc;
    const Walk walk = plan_walk(p, p->sweep, gfull, 1, 1, dppf_walk::kOnDemandReducing, 28.0 * kM);
    if (!rows_fit(p, grid, walk)) return DPPF_ELIMIT;
    shape->grid = grid;
    shape->walk = walk;
    hipLaunchKernelGGL(kern, dim3(grid), dim3(kBlock), 0, s, p->sweep.dev, walk, p->T, (float* const*)(xd),
                       (float* const*)(ad), (float* const*)(sd), (const float* const*)(gd), hp, p->partials,
                       p->partials_rows);
  })
  HIP_TRY(hipGetLastError());
  return DPPF_OK;
}

}  // namespace dppf_detail
