// Sweep 1 of the round for M <= 16 without a folded step: the average (kept in registers, optionally
// stored) and the squared distances to it.  Pure reads unless the average is stored.
#include "dppf_internal.h"

namespace dppf_detail {
namespace {

template <int XBAR, bool NORMS>
int launch(dppf_plan* p, const void** xp, const void** xbarp, KeepPolicy keep, GridShape* shape, hipStream_t s) {
  float* const* x = (float* const*)(xp);
  float* const* xb = (float* const*)(xbarp);
  DPPF_SWITCH_M(p->M, {
    constexpr int kU = unroll_plain(kM);
    auto kern = k_sweep1<kM, kU, false, XBAR, NORMS>;
    int grid = 0, gfull = 0;
    const int rc = grid_for(p, p->sweep, kern, 1, 1, XBAR == 1 ? kBlocksPerCUReadWrite : kBlocksPerCUReadOnly, 0,
                            &gfull, &grid);
    if (rc) return rc;
    const Walk walk = plan_walk(p, p->sweep, gfull, 1, 1, dppf_walk::kEvenSplit, 4.0 * kM);
    if (NORMS && !rows_fit(p, grid, walk)) return DPPF_ELIMIT;
    if (shape) {
      shape->grid = grid;
      shape->walk = walk;
    }
    hipLaunchKernelGGL(kern, dim3(grid), dim3(kBlock), 0, s, p->sweep.dev, walk, p->T, x, nullptr, nullptr, xb, 0.f,
                       0.f, 0.f, p->partials, p->partials_rows, keep_from_tile(p, keep));
  })
  HIP_TRY(hipGetLastError());
  return DPPF_OK;
}

}  // namespace

int launch_reduce(dppf_plan* p, const void** xp, const void** xbarp, bool store_avg, bool norms, KeepPolicy keep,
                  GridShape* shape, hipStream_t s) {
  if (store_avg && norms) return launch<1, true>(p, xp, xbarp, keep, shape, s);
  if (store_avg) return launch<1, false>(p, xp, xbarp, keep, shape, s);
  if (norms) return launch<0, true>(p, xp, nullptr, keep, shape, s);
  return DPPF_EINVAL;
}

}  // namespace dppf_detail
