// Streaming kernels for any number of workers that read a STORED average: used beyond 39 workers,
// by the variants of the round that have no LDS-staged form, and by dppf_replica_mean /
// dppf_dist_norms with a given average.  They walk the list of kStepTileElems-element tiles.
#include "dppf_internal.h"

namespace dppf_detail {
namespace {
size_t column_sums_bytes(int M) { return sizeof(double) * kWaves * (static_cast<size_t>(M) + 1); }
}  // namespace

int launch_mean_any(dppf_plan* p, const void** xp, const void** xbarp, hipStream_t s) {
  int grid = 0, gfull = 0;
  const int rc = grid_for(p, p->step, k_mean_any, 1, 1, kBlocksPerCUReadOnly, 0, &gfull, &grid);
  if (rc) return rc;
  const Walk walk = plan_walk(p, p->step, gfull, 1, 1, dppf_walk::kEvenSplit, 0.0);
  hipLaunchKernelGGL(k_mean_any, dim3(grid), dim3(kBlock), 0, s, p->step.dev, walk, p->M, p->T, (float* const*)(xp),
                     (float* const*)(xbarp));
  HIP_TRY(hipGetLastError());
  return DPPF_OK;
}

int launch_norms_any(dppf_plan* p, const void** xp, const void** xbarp, GridShape* shape, hipStream_t s) {
  int grid = 0, gfull = 0;
  const size_t lds = column_sums_bytes(p->M);
  const int rc = grid_for(p, p->step, k_norms_any, 1, 1, kBlocksPerCUReadOnly, lds, &gfull, &grid);
  if (rc) return rc;
  const Walk walk = plan_walk(p, p->step, gfull, 1, 1, dppf_walk::kEvenSplit, 0.0);
  if (!rows_fit(p, grid, walk)) return DPPF_ELIMIT;
  shape->grid = grid;
  shape->walk = walk;
  hipLaunchKernelGGL(k_norms_any, dim3(grid), dim3(kBlock), lds, s, p->step.dev, walk, p->M, p->T,
                     (float* const*)(xp), (const float* const*)(xbarp), p->partials, p->partials_rows);
  HIP_TRY(hipGetLastError());
  return DPPF_OK;
}

int launch_update_any(dppf_plan* p, const void** xp, const void** xbarp, const void** sump, bool exact, float k2,
                      hipStream_t s) {
  int grid = 0, gfull = 0, rc;
  auto kern = exact ? k_update_any<true> : k_update_any<false>;
  if ((rc = grid_for(p, p->step, kern, 1, 1, kBlocksPerCUReadWrite, 0, &gfull, &grid))) return rc;
  const Walk walk = plan_walk(p, p->step, gfull, 1, 1, dppf_walk::kOnDemand, 8.0 * p->M + (exact ? 8.0 : 4.0));
  hipLaunchKernelGGL(kern, dim3(grid), dim3(kBlock), 0, s, p->step.dev, walk, p->M, p->T, (float* const*)(xp),
                     (const float* const*)(xbarp), (const float* const*)(sump), p->coef, k2);
  HIP_TRY(hipGetLastError());
  return DPPF_OK;
}

int launch_unit_sum_any(dppf_plan* p, const void** xp, const void** xbarp, const void** sump, hipStream_t s) {
  int grid = 0, gfull = 0;
  const int rc = grid_for(p, p->step, k_unit_sum_any, 1, 1, kBlocksPerCUReadOnly, 0, &gfull, &grid);
  if (rc) return rc;
  const Walk walk = plan_walk(p, p->step, gfull, 1, 1, dppf_walk::kEvenSplit, 0.0);
  hipLaunchKernelGGL(k_unit_sum_any, dim3(grid), dim3(kBlock), 0, s, p->step.dev, walk, p->M, p->T,
                     (float* const*)(xp), (const float* const*)(xbarp), p->coef, (float* const*)(sump));
  HIP_TRY(hipGetLastError());
  return DPPF_OK;
}

int launch_seq_any(dppf_plan* p, const void** xp, const void** xcp, const void** refp, bool ref_is_consensus,
                   bool write, float pull, GridShape* shape, hipStream_t s) {
  const float keep = static_cast<float>(1.0 - static_cast<double>(pull));
  int grid = 0, gfull = 0, rc;
  auto kern = ref_is_consensus ? (write ? k_seq_any<1, true> : k_seq_any<1, false>)
                               : (write ? k_seq_any<2, true> : k_seq_any<2, false>);
  const size_t lds = write ? 0 : column_sums_bytes(p->M);
  if ((rc = grid_for(p, p->step, kern, 1, 1, write ? kBlocksPerCUReadWrite : kBlocksPerCUReadOnly, lds, &gfull,
                     &grid)))
    return rc;
  const Walk walk = plan_walk(p, p->step, gfull, 1, 1, write ? dppf_walk::kOnDemand : dppf_walk::kEvenSplit,
                              8.0 * p->M + 8.0);
  if (!write) {
    if (!rows_fit(p, grid, walk)) return DPPF_ELIMIT;
    shape->grid = grid;
    shape->walk = walk;
  }
  hipLaunchKernelGGL(kern, dim3(grid), dim3(kBlock), lds, s, p->step.dev, walk, p->M, p->T, (float* const*)(xp),
                     (const float* const*)(xcp), (const float* const*)(refp), pull, keep, p->coef, p->partials,
                     p->partials_rows);
  HIP_TRY(hipGetLastError());
  return DPPF_OK;
}

}  // namespace dppf_detail
